// k-means update step (paper Sec. 4.1: the centroid is the mean of its group).
//
// The mean is defined with a fixed summation order - members in token order, fp64 -
// so that the result does not depend on scheduling.  Two kernels:
//   rank:  a stable counting sort of the token indices of one unit by cluster id
//          (16 wavefronts, each histogramming and then placing its own contiguous range
//          of tokens, ballot-built peer masks keeping equal ids in token order);
//   mean:  one wavefront per centroid adds its members in fp64, divides by the count, rounds
//          to fp32 and then to bf16: in token order for short lists, in interleaved partial
//          sums for long ones (four per wavefront; the longest lists are spread over the
//          wavefronts of the block) when a test on the members' exponents shows that no
//          addition can round (then every order gives the same bits).
//          A group without members keeps its previous centroid.
// Also here: the residual pass that turns one smoothing stage's output into the next one's
// input (Eq. 5 on whole tensors, result rounded to bf16).
#include "qvg_internal.hpp"

namespace qvg {

constexpr int kRankThreads = 1024;
constexpr int kRankWaves = kRankThreads / 64;      // the tokens of a unit are split into 16 ranges
constexpr int kRankKeep = 8;                        // ids a lane keeps in registers between passes
constexpr int kRankK = kMaxClusters;                // histogram width

// Stable counting sort of token indices by cluster id, one workgroup per unit.
// Wavefront w owns the w-th contiguous range of tokens: it histograms the range, and after
// the scan (start of cluster k = tokens of lower clusters + tokens of k in earlier ranges) it
// places the range 64 tokens at a time.  Inside a step, lanes with equal ids are ranked by
// lane number (ballot-built peer masks), so equal ids keep their token order.
template <bool WIDE>                       // 16-bit ids (more than 256 centroids)
__global__ __launch_bounds__(kRankThreads)
void kmeans_rank_kernel(UpdateArgs a) {
    __shared__ int cnt[kRankWaves][kRankK];   // histogram per range, then running cursor
    __shared__ int total[kRankK];
    const int h = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int K = a.K;
    const int64_t N = a.n_tokens;
    const int64_t id0 = (int64_t)h * a.ids_stride * a.ids_step + a.ids_off;   // token n at element id0 + n * step
    const int64_t step = a.ids_step;
    auto id_of = [&](int64_t n) { return (int)load_id(a.ids, id0 + n * step, WIDE ? 1 : 0); };
    int32_t *perm = a.perm + (int64_t)h * N;
    int32_t *offs = a.offsets + (int64_t)h * (K + 1);

    const int Kp = (K + 63) & ~63;            // only the first Kp columns of the histograms are used
    for (int k = lane; k < Kp; k += 64) cnt[w][k] = 0;
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
            if (i < steps && n < end) { id = id_of(n); if (id >= K) id = -1; }
            kept[i] = id;
        }
#pragma unroll
        for (int i = 0; i < kRankKeep; ++i) if (kept[i] >= 0) atomicAdd(&cnt[w][kept[i]], 1);
    } else {
        for (int64_t n = beg + lane; n < end; n += 64) { const int id = id_of(n); if (id < K) atomicAdd(&cnt[w][id], 1); }
    }
    __syncthreads();
    if (tid < kRankK) {
        int t = 0;
        if (tid < K) for (int r = 0; r < kRankWaves; ++r) t += cnt[r][tid];
        total[tid] = t;
    }
    __syncthreads();
    constexpr int kPerLane = kRankK / 64;
    if (tid < 64) {                       // exclusive scan of total[0..kRankK-1] by one wavefront
        int v[kPerLane], run = 0;
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) { v[i] = total[lane * kPerLane + i]; run += v[i]; }
        int incl = run;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int o = __shfl_up(incl, off, 64);
            if (lane >= off) incl += o;
        }
        int start = incl - run;
#pragma unroll
        for (int i = 0; i < kPerLane; ++i) { total[lane * kPerLane + i] = start; start += v[i]; }
    }
    __syncthreads();
    if (tid < Kp) {
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
    if (!keep && beg + lane < end) { nxt = id_of(beg + lane); if (nxt >= K) nxt = -1; }
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
            if (nn < end) { nxt = id_of(nn); if (nxt >= K) nxt = -1; }
        }
        const bool valid = id >= 0;
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (int b = 0; b < 9; ++b) {
            if (b == 8 && !WIDE) break;                             // the ninth bit only with 16-bit ids
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

constexpr int kMeanThreads = 256;           // 4 wavefronts
constexpr int kMeanWaves = kMeanThreads / 64;
constexpr int kMeanParallelMin = 96;        // member lists at least this long try the order-free path
constexpr int kMeanCoopMin = 192;           // lists at least this long are summed by the whole block
                                            // (with one centroid per block: every order-free list)
constexpr int kMeanSmallGrid = 2048;        // up to this many centroids in a launch: one block each

typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, a), __builtin_bit_cast(ushort2_t, b)));
}
__device__ __forceinline__ uint32_t pk_min_u16(uint32_t a, uint32_t b) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_min(__builtin_bit_cast(ushort2_t, a), __builtin_bit_cast(ushort2_t, b)));
}

// Order-free partial sums of a member list: the wavefront takes the groups of 64 members
// first, first + step, .. of perm[beg .. end); lane = member slot (4) x 8 channels, 8 rows in
// flight per lane (ROWS = 16 where registers do not matter).  s: the lane's partial sums of its 8 channels; amax / amin: per 16-bit half the
// largest magnitude bits and the smallest non-zero magnitude bits minus one (0xffff: none).
template <int ROWS>
__device__ __forceinline__ void mean_partial(const bf16_t *xb, int64_t stride_token, const int32_t *perm, int beg,
                                             int end, int first, int step, int lane, double s[8], uint32_t amax[4],
                                             uint32_t amin[4]) {
    const int slot = lane >> 4;
    constexpr bool AHEAD = ROWS > 8;       // member indices requested a group ahead (two more registers)
    int base = beg + 64 * first;
    int nxt = (AHEAD && base + lane < end) ? perm[base + lane] : 0;
    for (; base < end; base += 64 * step) {
        int mine;                                                        // 64 member indices, one coalesced load
        if (AHEAD) {
            mine = nxt;
            const int nb = base + 64 * step;
            nxt = (nb + lane < end) ? perm[nb + lane] : 0;
        } else {
            mine = (base + lane < end) ? perm[base + lane] : 0;
        }
        const int cntm = (end - base < 64) ? end - base : 64;
        // slot s takes members s, s + 4, s + 8, .. of the group: ROWS rows in flight per lane
        for (int i0 = 0; 4 * i0 < cntm; i0 += ROWS) {
            uint4 row[ROWS];
#pragma unroll
            for (int i = 0; i < ROWS; ++i) {
                const int u = 4 * (i0 + i) + slot;
                const int idx = __shfl(mine, u & 63, 64);
                row[i] = (u < cntm) ? *reinterpret_cast<const uint4 *>(xb + (int64_t)idx * stride_token)
                                    : make_uint4(0u, 0u, 0u, 0u);
            }
#pragma unroll
            for (int i = 0; i < ROWS; ++i) {
                const uint32_t w[4] = {row[i].x, row[i].y, row[i].z, row[i].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    s[2 * e] += (double)bf16_lo(w[e]);
                    s[2 * e + 1] += (double)bf16_hi(w[e]);
                    const uint32_t mag = w[e] & 0x7fff7fffu;
                    const ushort2_t one = {1, 1};
                    amax[e] = pk_max_u16(amax[e], mag);
                    amin[e] = pk_min_u16(amin[e], __builtin_bit_cast(uint32_t, (ushort2_t)(__builtin_bit_cast(ushort2_t, mag) - one)));   // zero -> 0xffff
                }
            }
        }
    }
}

// no partial sum of n members can round in fp64 when ceil(log2 n) + 8 + emax - emin <= 53; mx /
// mn: the packed largest / smallest-non-zero-minus-one magnitude bits of two channels
__device__ __forceinline__ bool mean_exact(uint32_t mx, uint32_t mn, int lg) {
    bool ok = true;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
        const uint32_t big = (mx >> (16 * hf)) & 0xffffu, small1 = (mn >> (16 * hf)) & 0xffffu;
        if (small1 == 0xffffu) continue;                     // no non-zero member in this channel: the sum is zero
        const int eb = (int)(big >> 7) > 1 ? (int)(big >> 7) : 1;
        const int es = (int)((small1 + 1u) >> 7) > 1 ? (int)((small1 + 1u) >> 7) : 1;
        if (lg + 8 + eb - es > 53) ok = false;
    }
    return ok;
}

// the defining order: members in token order, two channels per lane, 16 rows in flight
__device__ __forceinline__ void mean_token_order(const bf16_t *xu, int64_t stride_token, const int32_t *perm, int beg,
                                                 int end, int lane, bf16_t *out) {
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
                    ? *reinterpret_cast<const uint32_t *>(xb + (int64_t)idx * stride_token) : 0u;
            }
#pragma unroll
            for (int u = 0; u < 16; ++u)
                if (u0 + u < cntm) { s0 += (double)bf16_lo(wv[u]); s1 += (double)bf16_hi(wv[u]); }
        }
    }
    const double c = (double)(end - beg);
    const float m0 = (float)(s0 / c), m1 = (float)(s1 / c);
    *reinterpret_cast<uint32_t *>(out + lane * 2) = pack_bf16x2(m0, m1);
}

// One wavefront per centroid, CPB = four centroids per block (or CPB = 1, see below).  The defined result is the fp64 sum of
// the members in token order.  Short lists are summed exactly like that.  A long list is
// latency-bound that way (one dependent fp64 add per member), so it is first summed in
// interleaved partial sums, which give the same number whenever no addition rounds: every member
// is an integer multiple of 2^(emin-134) and every partial sum is below n * 256 * 2^(emax-134),
// with emin / emax the smallest / largest exponent field among the non-zero members of the
// channel, so if
//     ceil(log2 n) + 8 + emax - emin <= 53
// all partial sums of any order are exact in fp64.  The exponents are tracked alongside (packed
// 16-bit min / max of the magnitudes' bit patterns); a centroid with a channel that fails the
// test is summed again in token order.  Lists of medium length use the four member slots of their
// own wavefront; the longest ones (one cluster can hold a large share of a unit's tokens, e.g.
// in the later smoothing stages) are split over all wavefronts of the block, whose partial
// results meet in LDS.  Four wavefronts per block and at most 80 registers (the few values that
// spill are touched once per block-wide list) keep six wavefronts per SIMD resident, which is what
// the common case of many short lists lives on; eight wavefronts per block sum the longest lists
// faster and everything else slower.  A launch with few centroids (one chunk of a few heads) cannot
// fill the chip anyway and is a chain of dependent loads: there a block has ONE centroid (CPB = 1),
// every list long enough for the order-free path is spread over the block's four wavefronts, and
// 16 rows are in flight per lane (ROWS = 16: no occupancy to protect).
template <int CPB, int ROWS>
__global__ __launch_bounds__(kMeanThreads, CPB == 1 ? 2 : 6)
void kmeans_mean_kernel(UpdateArgs a) {
    constexpr int kCoopMin = CPB == 1 ? kMeanParallelMin : kMeanCoopMin;
    __shared__ double part[kMeanWaves][kHeadDim];
    __shared__ uint32_t pmx[kMeanWaves][kHeadDim / 2], pmn[kMeanWaves][kHeadDim / 2];
    const int h = blockIdx.y, lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int j0 = blockIdx.x * CPB;
    const int j = j0 + wave;
    const int K = a.K;
    const int64_t N = a.n_tokens;
    const int32_t *offs = a.offsets + (int64_t)h * (K + 1);
    const int32_t *perm = a.perm + (int64_t)h * N;
    const bf16_t *xu = a.x + (int64_t)h * a.stride_head;
    const int slot = lane >> 4, c8 = lane & 15;
    // the block's list boundaries with one load per wavefront (lane i: start of centroid j0 + i);
    // used after the wavefront's own list
    const int myoff = (lane <= CPB && j0 + lane <= K) ? offs[j0 + lane] : 0;

    // ---- the wavefront's own centroid, unless its list is left to the whole block ----
    if (wave < CPB && j < K) {
        const int beg = offs[j], end = offs[j + 1];                      // wave-uniform: scalar loads
        const int64_t co = ((int64_t)h * K + j) * kHeadDim;
        if (end == beg) {
            *reinterpret_cast<uint32_t *>(a.cent_out + co + lane * 2) = *reinterpret_cast<const uint32_t *>(a.cent_prev + co + lane * 2);
        } else if (end - beg < kCoopMin) {
            bool done = false;
            if (CPB > 1 && end - beg >= kMeanParallelMin) {
                double s[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) s[i] = 0.0;
                uint32_t amax[4] = {0u, 0u, 0u, 0u}, amin[4] = {~0u, ~0u, ~0u, ~0u};
                mean_partial<ROWS>(xu + c8 * 8, a.stride_token, perm, beg, end, 0, 1, lane, s, amax, amin);
                // the four slots hold partial results of the same channels: lanes l, l^16, l^32, l^48
                int lg = 0;
                while ((1 << lg) < end - beg) ++lg;                          // ceil(log2 n)
                bool ok = true;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    uint32_t mx = amax[e], mn = amin[e];
#pragma unroll
                    for (int off = 16; off <= 32; off <<= 1) {
                        mx = pk_max_u16(mx, __shfl_xor(mx, off, 64));
                        mn = pk_min_u16(mn, __shfl_xor(mn, off, 64));
                    }
                    ok = ok && mean_exact(mx, mn, lg);
                }
                if (__all(ok)) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        s[i] += __shfl_xor(s[i], 16, 64);
                        s[i] += __shfl_xor(s[i], 32, 64);
                    }
                    if (slot == 0) {
                        const double c = (double)(end - beg);
                        float m[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i) m[i] = (float)(s[i] / c);
                        *reinterpret_cast<uint4 *>(a.cent_out + co + c8 * 8) = pack_bf16x8(m);
                    }
                    done = true;
                }
            }
            if (!done) mean_token_order(xu, a.stride_token, perm, beg, end, lane, a.cent_out + co);
        }
    }

    // ---- the block's longest lists, one after the other, by all wavefronts (every wavefront of
    // the block takes the same branches: the list lengths are read by all of them) ----
    const int mylen = __shfl_down(myoff, 1, 64) - myoff;                 // all lanes take part in the exchange
    const uint64_t coop = __ballot(lane < CPB && j0 + lane < K && mylen >= kCoopMin);   // the same in every wavefront
    for (uint64_t todo = coop; todo; todo &= todo - 1) {
        const int t = __builtin_ctzll(todo);
        const int jt = j0 + t;
        const int beg = __shfl(myoff, t, 64), end = __shfl(myoff, t + 1, 64);
        double s[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) s[i] = 0.0;
        uint32_t amax[4] = {0u, 0u, 0u, 0u}, amin[4] = {~0u, ~0u, ~0u, ~0u};
        mean_partial<ROWS>(xu + c8 * 8, a.stride_token, perm, beg, end, wave, kMeanWaves, lane, s, amax, amin);
#pragma unroll
        for (int i = 0; i < 8; ++i) {          // harmless if an addition rounds: then the result is discarded
            s[i] += __shfl_xor(s[i], 16, 64);
            s[i] += __shfl_xor(s[i], 32, 64);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
#pragma unroll
            for (int off = 16; off <= 32; off <<= 1) {
                amax[e] = pk_max_u16(amax[e], __shfl_xor(amax[e], off, 64));
                amin[e] = pk_min_u16(amin[e], __shfl_xor(amin[e], off, 64));
            }
        }
        if (slot == 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) part[wave][c8 * 8 + i] = s[i];
#pragma unroll
            for (int e = 0; e < 4; ++e) { pmx[wave][c8 * 4 + e] = amax[e]; pmn[wave][c8 * 4 + e] = amin[e]; }
        }
        __syncthreads();
        if (wave == t) {                      // the centroid's own wavefront (t < CPB): channels 2*lane, 2*lane+1
            double s0 = 0.0, s1 = 0.0;
            uint32_t mx = 0u, mn = ~0u;
#pragma unroll
            for (int w = 0; w < kMeanWaves; ++w) {
                s0 += part[w][2 * lane];
                s1 += part[w][2 * lane + 1];
                mx = pk_max_u16(mx, pmx[w][lane]);
                mn = pk_min_u16(mn, pmn[w][lane]);
            }
            int lg = 0;
            while ((1 << lg) < end - beg) ++lg;
            const int64_t co = ((int64_t)h * K + jt) * kHeadDim;
            if (__all(mean_exact(mx, mn, lg))) {
                const double c = (double)(end - beg);
                *reinterpret_cast<uint32_t *>(a.cent_out + co + lane * 2) = pack_bf16x2((float)(s0 / c), (float)(s1 / c));
            } else {
                mean_token_order(xu, a.stride_token, perm, beg, end, lane, a.cent_out + co);
            }
        }
        __syncthreads();                      // the partial results are overwritten by the next list
    }
}

// Residual for the next smoothing stage: 16 lanes per token, 8 channels each.
__global__ __launch_bounds__(256)
void residual_kernel(ResidualArgs a) {
    const int h = blockIdx.y;
    const int64_t n = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const int c8 = threadIdx.x & 15;
    if (n >= a.n_tokens) return;
    int id = (int)load_id(a.ids, ((int64_t)h * a.ids_stride + n) * a.ids_step + a.ids_off, a.id_wide);
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
    if (a.id_wide) hipLaunchKernelGGL(kmeans_rank_kernel<true>, dim3((unsigned)a.H), dim3(kRankThreads), 0, s, a);
    else hipLaunchKernelGGL(kmeans_rank_kernel<false>, dim3((unsigned)a.H), dim3(kRankThreads), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if ((int64_t)a.K * a.H <= kMeanSmallGrid) {
        hipLaunchKernelGGL((kmeans_mean_kernel<1, 16>), dim3((unsigned)a.K, (unsigned)a.H), dim3(kMeanThreads), 0, s, a);
    } else {
        dim3 grid((unsigned)((a.K + kMeanWaves - 1) / kMeanWaves), (unsigned)a.H);
        hipLaunchKernelGGL((kmeans_mean_kernel<kMeanWaves, 8>), grid, dim3(kMeanThreads), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace qvg
