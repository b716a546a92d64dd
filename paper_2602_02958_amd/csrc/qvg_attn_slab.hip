// Attention over the compressed cache with the decoded tiles shared by all query blocks.
//
// The fused kernels (qvg_attn.hip) decode every 64-token tile once per workgroup of 256 queries:
// with n_q queries per unit the dequantization of Eq. 7 is repeated ceil(n_q / 256) times, and it
// is what bounds them (vector instructions, not the matrix cores).  When the caller lends a
// workspace, the same work is split at the point where those kernels hand a decoded tile to the
// contractions:
//   slab_decode_kernel   decodes each tile of a slab of chunks ONCE per unit and writes the two
//                        operand images the contractions read: K_hat row-major bf16 [64][128], V_hat
//                        transposed f16 [128][64] with the token permutation of the PV contraction
//                        (the values are exactly those the fused kernels put into LDS);
//   attn_slab_kernel     256 queries per workgroup as before; per tile it copies the two images
//                        (32 KB) into LDS and runs the same S^T = K Q^T, online soft-max and
//                        O^T += V^T P steps.
// A slab is as many whole chunks as the workspace holds; the running soft-max state (maximum,
// normaliser, unnormalised output, fp32) of every query is carried from slab to slab in the
// workspace, so the full-precision cache is never materialised beyond one slab.
#include "qvg_attn_tiles.hpp"

namespace qvg {

constexpr int kImgElems = kAtKv * kHeadDim;             // 16-bit elements of one operand image (16 KB)
constexpr int kStateFloats = 66;                        // per thread: 64 output values, maximum, normaliser

struct SlabArgs {
    uint16_t *kimg, *vimg;     // [H][tiles_cap][kImgElems]
    int64_t tiles_cap;         // image slots per unit
    int c0;                    // first chunk of the slab
    int n_tiles;               // tiles of the slab (every one holds at least one token)
    int tpc;                   // tiles per chunk = ceil(chunk_len / 64)
    float *state;              // [workgroup][kStateFloats][512] running state, or nullptr (single slab)
    int first, last;           // first / last slab of the call
};

// tile `i` of the slab (i may be past the end: then invalid)
__device__ __forceinline__ Tile slab_tile(const AttnArgs &a, const SlabArgs &sl, int i) {
    Tile t;
    const int c = i / sl.tpc;
    t.chunk = sl.c0 + c;
    const int64_t b = (int64_t)t.chunk * a.chunk_len;
    t.t0 = (int)(b + (int64_t)(i - c * sl.tpc) * kAtKv);
    t.cend = (int)((b + a.chunk_len < a.n_kv) ? b + a.chunk_len : a.n_kv);
    t.valid = i < sl.n_tiles;
    if (!t.valid) { t.chunk = sl.c0; t.t0 = 0; t.cend = 0; }
    return t;
}

// ---------------------------------------------------------------------------------------------
// Decode a run of tiles of one unit's K and V into the operand images.  512 threads: thread
// (tp, c8) has tokens 2 tp, 2 tp + 1 and channels 8 c8 .. 8 c8 + 7 of both sides, as in the fused
// kernels.  K rows go straight to memory (16 lanes cover a 256-byte row); V is transposed through
// LDS.  Tokens past the end of a chunk decode to zero.
// ---------------------------------------------------------------------------------------------
template <int TM, int SM>
struct TileRaw { Raw<TM, SM> k, v; uint4 rp[2]; };

// Two workgroups per CU (at most 128 registers) for the instances with one smoothing stage and a
// compile-time round count: the kernel is a chain of small dependent loads and lives on occupancy.
template <int T_, int SM, int FMT, bool ROPE>
__global__ __launch_bounds__(kAtThreads, (T_ > 0 && SM == 1) ? 4 : 2)
void slab_decode_kernel(AttnArgs a, SlabArgs sl, int run) {
    constexpr int TM = T_ > 0 ? T_ : kMaxStages;
    __shared__ __align__(16) uint16_t Vt[kVtElems];                     // [128][72] f16, transposed, swizzled (below)
    const int h = blockIdx.y;
    const int i0 = (int)blockIdx.x * run;
    const int i1 = (i0 + run < sl.n_tiles) ? i0 + run : sl.n_tiles;
    const int tid = threadIdx.x;
    const int T = T_ > 0 ? T_ : a.T, B = a.B, K = a.K;
    const int S = SM > 0 ? SM : a.S;
    const int G = kHeadDim / B;

    CacheSide ks, vs;
    constexpr int kCodeBytes = (FMT & kFmtInt4) ? 64 : 32, kScaleBytes = (FMT & kFmtE4M3) ? 1 : 2;
    ks.ids = a.k_ids + (int64_t)h * a.kv_stride * S * (a.id_wide ? 2 : 1);  ks.codes = a.k_codes + (int64_t)h * a.kv_stride * T * kCodeBytes;
    ks.scales = reinterpret_cast<const uint8_t *>(a.k_scales) + (int64_t)h * a.kv_stride * T * G * kScaleBytes;
    ks.cent = a.k_cent + (int64_t)h * a.chunk_stride * S * K * kHeadDim;
    ks.wide = vs.wide = a.id_wide;
    vs.ids = a.v_ids + (int64_t)h * a.kv_stride * S * (a.id_wide ? 2 : 1);  vs.codes = a.v_codes + (int64_t)h * a.kv_stride * T * kCodeBytes;
    vs.scales = reinterpret_cast<const uint8_t *>(a.v_scales) + (int64_t)h * a.kv_stride * T * G * kScaleBytes;
    vs.cent = a.v_cent + (int64_t)h * a.chunk_stride * S * K * kHeadDim;

    const int c8 = tid & 15, tp = tid >> 4;
    const int g = (c8 * 8) / B;
    const int tok = 2 * tp;
    // position of the token pair in a transposed V row (the order in which a lane's soft-max
    // values feed the PV contraction): token 16 s + 8 a + 4 hh + e sits at 16 s + 8 hh + 4 a + e
    const int v_pos = 16 * (tok >> 4) + 8 * ((tok >> 2) & 1) + 4 * ((tok >> 3) & 1) + (tok & 3);
    uint16_t *kimg = sl.kimg + (int64_t)h * sl.tiles_cap * kImgElems;
    uint16_t *vimg = sl.vimg + (int64_t)h * sl.tiles_cap * kImgElems;

    uint32_t idk[2], idv[2];
    auto fetch = [&](const Tile &t, TileRaw<TM, SM> &r) {            // ids of `t` are in idk / idv
        load_raw<T_, TM, SM, FMT>(ks, t, tp, c8, T, G, g, K, S, idk, r.k);
        load_raw<T_, TM, SM, FMT>(vs, t, tp, c8, T, G, g, K, S, idv, r.v);
        if (ROPE) load_rope(a.rope, t, tp, c8, r.rp);
    };
    // decode the tile held in r (both sides) and write its two images; `next` is called as soon as
    // r has been consumed: it requests the following tile into the same registers, so that its
    // loads are in flight during the transposition (with two workgroups per CU the other one's
    // work hides the rest of their latency)
    auto emit = [&](int i, TileRaw<TM, SM> &r, auto next) {
        float accA[8], accB[8];
        dequant2x8<T_, TM, SM, FMT>(r.k, T, accA, accB);
        if (ROPE) { rope_rotate8(accA, r.rp[0]); rope_rotate8(accB, r.rp[1]); }
        uint16_t *kt = kimg + (int64_t)i * kImgElems;
        *reinterpret_cast<uint4 *>(kt + (tok + 0) * kHeadDim + c8 * 8) = pack_bf16x8(accA);
        *reinterpret_cast<uint4 *>(kt + (tok + 1) * kHeadDim + c8 * 8) = pack_bf16x8(accB);
        dequant2x8<T_, TM, SM, FMT>(r.v, T, accA, accB);
        next();
        // rows 8 c8 .. 8 c8 + 7; the 16-byte group of a row is XOR-ed with (row / 8) & 7 so that the 16
        // lanes that write the same column of 16 different row groups spread over the banks
        uint16_t *vt = Vt + (((v_pos >> 3) ^ (c8 & 7)) * 8 + (v_pos & 7));
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            // round to bf16 (the decoder's output), then to f16 (exact in range): channels e, e+1
            const uint32_t pa = pack_bf16x2(accA[e], accA[e + 1]);
            const uint32_t pb = pack_bf16x2(accB[e], accB[e + 1]);
            *reinterpret_cast<uint32_t *>(vt + (c8 * 8 + e) * kVtPitch) = pack_f16x2_rtz(bf16_lo(pa), bf16_lo(pb));
            *reinterpret_cast<uint32_t *>(vt + (c8 * 8 + e + 1) * kVtPitch) = pack_f16x2_rtz(bf16_hi(pa), bf16_hi(pb));
        }
        __syncthreads();
        uint16_t *vo = vimg + (int64_t)i * kImgElems;
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int p = tid + k * kAtThreads;                          // 16-byte piece: row p / 8, group p % 8
            *reinterpret_cast<uint4 *>(vo + p * 8) =
                *reinterpret_cast<const uint4 *>(Vt + (p >> 3) * kVtPitch + (((p & 7) ^ ((p >> 6) & 7)) * 8));
        }
        __syncthreads();                                                 // Vt is rewritten by the next tile
    };

    if (i0 >= i1) return;                                                // uniform
    // raw data one tile ahead (requested as soon as the registers are free), ids two tiles ahead
    TileRaw<TM, SM> r;
    Tile t = slab_tile(a, sl, i0);
    load_ids(ks, t, tp, S, a.id_wide, idk);
    load_ids(vs, t, tp, S, a.id_wide, idv);
    fetch(t, r);
    Tile tn = slab_tile(a, sl, i0 + 1 < i1 ? i0 + 1 : sl.n_tiles);
    load_ids(ks, tn, tp, S, a.id_wide, idk);
    load_ids(vs, tn, tp, S, a.id_wide, idv);
    for (int i = i0; i < i1; ++i) {
        emit(i, r, [&]() {
            fetch(tn, r);                                                // tile i + 1 (its ids arrived an iteration ago)
            tn = slab_tile(a, sl, i + 2 < i1 ? i + 2 : sl.n_tiles);
            load_ids(ks, tn, tp, S, a.id_wide, idk);
            load_ids(vs, tn, tp, S, a.id_wide, idv);
        });
    }
}

// ---------------------------------------------------------------------------------------------
// S^T = K Q^T, online soft-max (base 2), O^T += V^T P on one tile held in LDS (layouts of the
// fused kernels: K [64][136] bf16, V [128][72] f16 transposed, 16-byte groups of a row XOR-ed with
// 2 * (row / 32)).  ntile: tokens the tile holds (scores of the others are masked).
// ---------------------------------------------------------------------------------------------
// left: tokens of this tile the lane's query sees (only looked at when ql_mask is set: some query of
// the wavefront ends in or before this tile).
__device__ __forceinline__ void slab_tile_attend(const uint16_t *kt, const uint16_t *vt, const uint4 (&qa)[8], int col,
                                                 int half, int ntile, bool ql_mask, int left, float scale2,
                                                 floatx16_t (&O)[4], float &m, float &l) {
    floatx16_t S[2];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) S[nb][r] = 0.0f;
    {
        constexpr int kKAhead = 4;                                       // operand fragments in flight
        const uint16_t *arow = kt + col * kKtPitch + half * 8;
        auto kfrag = [&](int i) {
            return *reinterpret_cast<const bf16x8_t *>(arow + (i >> 3) * 32 * kKtPitch + (i & 7) * 16);
        };
        bf16x8_t kf[16];
#pragma unroll
        for (int i = 0; i < kKAhead; ++i) kf[i] = kfrag(i);
        __builtin_amdgcn_sched_group_barrier(0x100, kKAhead, 0);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            S[i >> 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                kf[i], __builtin_bit_cast(bf16x8_t, qa[i & 7]), S[i >> 3], 0, 0, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (i + kKAhead < 16) {
                kf[i + kKAhead] = kfrag(i + kKAhead);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        }
    }
    if (ntile < kAtKv) {                                                 // uniform: last tile of a chunk
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kv = nb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                if (kv >= ntile) S[nb][r] = -INFINITY;
            }
    }
    if (ql_mask) {                                                       // uniform
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kv = nb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                if (kv >= left) S[nb][r] = -INFINITY;
            }
    }
    float tmax = -INFINITY;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, S[nb][r]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64)) * scale2;               // the scale is positive: order kept
    const float m_new = fmaxf(m, tmax);
    if (__ballot(m_new > m)) {                                           // uniform: skip when no maximum moved
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
        for (int e = 0; e < 8; ++e)
            p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(S[st >> 1][(st & 1) * 8 + e], scale2, -m));
        pb[st] = make_uint4(pack_f16x2_rne(p[0], p[1]), pack_f16x2_rne(p[2], p[3]),
                            pack_f16x2_rne(p[4], p[5]), pack_f16x2_rne(p[6], p[7]));
        // the normaliser is the sum of the f16 probabilities the PV contraction uses
        l = sum_f16_pairs(pb[st], l);
    }
    {
        constexpr int kVAhead = 4;
        auto vfrag = [&](int i) {
            const int mb = i >> 2, st = i & 3;
            const int key = mb * 2;
            return *reinterpret_cast<const halfx8_t *>(vt + (mb * 32 + col) * kVtPitch + (((2 * st + half) ^ key) * 8));
        };
        halfx8_t vf[16];
#pragma unroll
        for (int i = 0; i < kVAhead; ++i) vf[i] = vfrag(i);
        __builtin_amdgcn_sched_group_barrier(0x100, kVAhead, 1);
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            O[i >> 2] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                vf[i], __builtin_bit_cast(halfx8_t, pb[i & 3]), O[i >> 2], 0, 0, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
            if (i + kVAhead < 16) {
                vf[i + kVAhead] = vfrag(i + kVAhead);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 1);
            }
        }
    }
}

// One workgroup = 8 wavefronts = 256 queries of one unit, over the tiles of one slab.
// QL: a prefix length per query (a.q_len): scores beyond the lane's prefix are masked in the tiles
// at or past the shortest prefix of the wavefront, and the workgroup stops at the longest prefix
// among its 256 queries.
template <bool QL>
__global__ __launch_bounds__(kAtThreads, 2)
void attn_slab_kernel(AttnArgs a, SlabArgs sl, int n_qblocks, int n_blocks, int blocks_per_xcd) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t *Kt = reinterpret_cast<uint16_t *>(smem);                  // [2][64][136] bf16
    uint16_t *Vt = Kt + 2 * kKtElems;                                   // [2][128][72] f16, transposed

    // the query blocks of one unit run on one XCD, whose L2 then serves the unit's images to all of them
    const int w = (int)(blockIdx.x % 8u) * blocks_per_xcd + (int)(blockIdx.x / 8u);
    if (w >= n_blocks) return;                                          // uniform, before any barrier
    const int h = w / n_qblocks;
    const int qblock = w - h * n_qblocks;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int64_t qrow = (int64_t)qblock * kAtQPerBlock + wave * 32 + col;
    const bool qvalid = qrow < a.n_q;

    uint4 qa[8];
    {
        const bf16_t *qp = a.q + ((int64_t)h * a.n_q + qrow) * kHeadDim + half * 8;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
            qa[kk] = qvalid ? *reinterpret_cast<const uint4 *>(qp + kk * 16) : make_uint4(0u, 0u, 0u, 0u);
    }
    floatx16_t O[4];
    float m = -INFINITY, l = 0.0f;
    float *st = sl.state ? sl.state + (int64_t)w * kStateFloats * kAtThreads + tid : nullptr;
    if (sl.first) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) O[mb][r] = 0.0f;
    } else {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) O[mb][r] = st[(mb * 16 + r) * kAtThreads];
        m = st[64 * kAtThreads];
        l = st[65 * kAtThreads];
    }
    const float scale2 = a.scale * 1.4426950408889634f;
    int qlen = 0x7fffffff, wmin = 0x7fffffff, wgmax = 0x7fffffff;
    if (QL) {
        __shared__ int bmax;
        if (tid == 0) bmax = 0;
        __syncthreads();
        const int nk = (int)a.n_kv;
        qlen = 0;
        if (qvalid) { const int v = a.q_len[qrow]; qlen = v < 0 ? 0 : (v > nk ? nk : v); }
        wmin = qvalid ? qlen : 0x7fffffff;
        int mx = qlen;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const int o = __shfl_xor(wmin, off, 64); wmin = o < wmin ? o : wmin;
            const int p = __shfl_xor(mx, off, 64); mx = p > mx ? p : mx;
        }
        if (lane == 0) atomicMax(&bmax, mx);
        __syncthreads();
        wgmax = bmax;
        wmin = __builtin_amdgcn_readfirstlane(wmin);
    }

    // a thread's four 16-byte pieces of a tile: K pieces tid, tid + 512 (row p / 16, group p % 16),
    // V pieces tid, tid + 512 (row p / 8, group p % 8, XOR-ed with the row's key in LDS)
    const uint16_t *kimg = sl.kimg + (int64_t)h * sl.tiles_cap * kImgElems + tid * 8;
    const uint16_t *vimg = sl.vimg + (int64_t)h * sl.tiles_cap * kImgElems + tid * 8;
    auto k_off = [&](int p) { return (p >> 4) * kKtPitch + (p & 15) * 8; };
    auto v_off = [&](int p) { const int row = p >> 3; return row * kVtPitch + (((p & 7) ^ ((row >> 5) * 2)) * 8); };
    const int koff[2] = {k_off(tid), k_off(tid + kAtThreads)};
    const int voff[2] = {v_off(tid), v_off(tid + kAtThreads)};
    // The pieces of a tile are requested two iterations before they go to LDS: two register sets,
    // used in turn, so that the park does not wait for them (requested one iteration ahead: 22.8
    // against 22.1 ms per cfg5 call).
    const int n = sl.n_tiles;                                           // >= 1
    auto clampt = [&](int i) { return i < n ? i : n - 1; };            // past the end: the last tile once more (never used)
    uint4 pa0, pa1, pa2, pa3, pb0, pb1, pb2, pb3;
#define QVG_SLAB_FETCH(s_, i_)                                                                    \
    {                                                                                             \
        const int ti_ = clampt(i_);                                                               \
        const uint16_t *kp_ = kimg + (int64_t)ti_ * kImgElems, *vp_ = vimg + (int64_t)ti_ * kImgElems; \
        s_##0 = *reinterpret_cast<const uint4 *>(kp_);                                            \
        s_##1 = *reinterpret_cast<const uint4 *>(kp_ + kAtThreads * 8);                           \
        s_##2 = *reinterpret_cast<const uint4 *>(vp_);                                            \
        s_##3 = *reinterpret_cast<const uint4 *>(vp_ + kAtThreads * 8);                           \
    }
#define QVG_SLAB_PARK(s_, buf_)                                                                   \
    {                                                                                             \
        uint16_t *kt_ = Kt + (buf_) * kKtElems, *vt_ = Vt + (buf_) * kVtElems;                    \
        *reinterpret_cast<uint4 *>(kt_ + koff[0]) = s_##0;                                        \
        *reinterpret_cast<uint4 *>(kt_ + koff[1]) = s_##1;                                        \
        *reinterpret_cast<uint4 *>(vt_ + voff[0]) = s_##2;                                        \
        *reinterpret_cast<uint4 *>(vt_ + voff[1]) = s_##3;                                        \
    }
    // one iteration's work on tile i in buffer buf; false when the loop ends here
    auto attend = [&](int i, int buf) -> bool {
        const Tile t = slab_tile(a, sl, i);
        if (QL && t.t0 >= wgmax) return false;                          // uniform: no query of the workgroup sees this tile or a later one
        const int ntile = (t.cend - t.t0 < kAtKv) ? t.cend - t.t0 : kAtKv;
        slab_tile_attend(Kt + buf * kKtElems, Vt + buf * kVtElems, qa, col, half, ntile, QL && t.t0 + kAtKv > wmin,
                         qlen - t.t0, scale2, O, m, l);
        return i + 1 < n;
    };
    // tile 0 parked; set a holds tile 1, set b tile 2.  After the work on tile i, tile i + 1 goes from
    // its set into the other buffer (nobody reads it in this iteration) and the set is refilled
    // with tile i + 3.  (Parking in the middle of the iteration, between the score contractions
    // and the soft-max, was slower: 22.5 against 22.1 ms per cfg5 call.)
    QVG_SLAB_FETCH(pa, 0);
    QVG_SLAB_PARK(pa, 0);
    QVG_SLAB_FETCH(pa, 1);
    QVG_SLAB_FETCH(pb, 2);
    __syncthreads();
    for (int i = 0; i < n; i += 2) {
        if (!attend(i, 0)) break;                                       // uniform
        QVG_SLAB_PARK(pa, 1);
        QVG_SLAB_FETCH(pa, i + 3);
        __syncthreads();
        if (!attend(i + 1, 1)) break;
        QVG_SLAB_PARK(pb, 0);
        QVG_SLAB_FETCH(pb, i + 4);
        __syncthreads();
    }
#undef QVG_SLAB_FETCH
#undef QVG_SLAB_PARK
    if (sl.last) {
        store_result(a, h, qrow, qvalid && (!QL || qlen > 0), qvalid, half, O, m, l);
    } else {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int r = 0; r < 16; ++r) st[(mb * 16 + r) * kAtThreads] = O[mb][r];
        st[64 * kAtThreads] = m;
        st[65 * kAtThreads] = l;
    }
}

// ---- host side ---------------------------------------------------------------------------------
template <int T_, int SM, int FMT>
static hipError_t launch_slab_decode_t(const AttnArgs &a, const SlabArgs &sl, hipStream_t s) {
    constexpr int kRun = 8;                                             // tiles per workgroup
    dim3 grid((unsigned)((sl.n_tiles + kRun - 1) / kRun), (unsigned)a.H);
    if (a.rope) hipLaunchKernelGGL((slab_decode_kernel<T_, SM, FMT, true>), grid, dim3(kAtThreads), 0, s, a, sl, kRun);
    else hipLaunchKernelGGL((slab_decode_kernel<T_, SM, FMT, false>), grid, dim3(kAtThreads), 0, s, a, sl, kRun);
    return hipGetLastError();
}

// instances with the round and stage counts fixed at compile time for the paper's forms, run-time
// counts for everything else
template <int FMT>
static hipError_t launch_slab_decode_f(const AttnArgs &a, const SlabArgs &sl, hipStream_t s) {
    if (a.S == 1) {
        if constexpr (FMT == 0) {
            switch (a.T) {
                case 1: return launch_slab_decode_t<1, 1, FMT>(a, sl, s);
                case 2: return launch_slab_decode_t<2, 1, FMT>(a, sl, s);
                case 3: return launch_slab_decode_t<3, 1, FMT>(a, sl, s);
                case 4: return launch_slab_decode_t<4, 1, FMT>(a, sl, s);
                default: break;
            }
            return launch_slab_decode_t<0, 1, FMT>(a, sl, s);
        } else {
            if (a.T == 1) return launch_slab_decode_t<1, 1, FMT>(a, sl, s);
            return launch_slab_decode_t<0, 1, FMT>(a, sl, s);
        }
    }
    if (a.T == 1 && a.S == 4 && !a.id_wide) return launch_slab_decode_t<1, 4, FMT>(a, sl, s);
    if (a.T == 1 && a.S == 2 && !a.id_wide) return launch_slab_decode_t<1, 2, FMT>(a, sl, s);
    return launch_slab_decode_t<0, 0, FMT>(a, sl, s);
}

static hipError_t launch_slab_decode(const AttnArgs &a, const SlabArgs &sl, hipStream_t s) {
    switch (a.fmt) {
        case 0: return launch_slab_decode_f<0>(a, sl, s);
        case kFmtE4M3: return launch_slab_decode_f<kFmtE4M3>(a, sl, s);
        case kFmtInt4: return launch_slab_decode_f<kFmtInt4>(a, sl, s);
        default: return launch_slab_decode_f<kFmtInt4 | kFmtE4M3>(a, sl, s);
    }
}

size_t attn_slab_state_bytes(int H, int64_t n_q) {
    const int64_t nqb = (n_q + kAtQPerBlock - 1) / kAtQPerBlock;
    return ((size_t)nqb * H * kStateFloats * kAtThreads * sizeof(float) + 255) / 256 * 256;
}
size_t attn_slab_chunk_bytes(int H, int64_t chunk_len) {
    const int64_t tpc = (chunk_len + kAtKv - 1) / kAtKv;
    return (size_t)H * tpc * 2 * kImgElems * sizeof(uint16_t);
}

// Whether the shared-tile path serves this call with this workspace: more than one query block
// per unit (else nothing is shared) and room for at least one chunk's tiles (plus the running
// state when the cache needs more than one slab).
bool attn_slab_applicable(const AttnArgs &a, const void *ws, size_t ws_bytes) {
    if (!ws || a.n_q <= kAtQPerBlock) return false;
    const size_t chunk = attn_slab_chunk_bytes(a.H, a.chunk_len);
    if (ws_bytes >= chunk * (size_t)a.n_chunks) return true;
    const size_t state = attn_slab_state_bytes(a.H, a.n_q);
    return ws_bytes >= state + chunk;
}

hipError_t launch_attn_slab(const AttnArgs &a, void *ws, size_t ws_bytes, hipStream_t s) {
    const int64_t tpc = (a.chunk_len + kAtKv - 1) / kAtKv;
    const size_t chunk = attn_slab_chunk_bytes(a.H, a.chunk_len);
    const bool single = ws_bytes >= chunk * (size_t)a.n_chunks;
    const size_t state = single ? 0 : attn_slab_state_bytes(a.H, a.n_q);
    int64_t slab_chunks = single ? a.n_chunks : (int64_t)((ws_bytes - state) / chunk);
    if (slab_chunks < 1 || tpc * slab_chunks > 0x7fffffff) return hipErrorInvalidValue;
    if (slab_chunks > a.n_chunks) slab_chunks = a.n_chunks;

    static LdsHighWater lds_limit = {};
    static LdsHighWater lds_limit_ql = {};
    hipError_t e = a.q_len ? ensure_dynamic_lds(reinterpret_cast<const void *>(&attn_slab_kernel<true>), kAtSmem, lds_limit_ql)
                           : ensure_dynamic_lds(reinterpret_cast<const void *>(&attn_slab_kernel<false>), kAtSmem, lds_limit);
    if (e != hipSuccess) return e;
    const int64_t nqb = (a.n_q + kAtQPerBlock - 1) / kAtQPerBlock;
    const int64_t nb = nqb * a.H;
    if (nb > 0x7fffffff - 8) return hipErrorInvalidValue;
    const int bpx = (int)((nb + 7) / 8);
    if ((int64_t)bpx * 8 > nb + 7) return hipErrorInvalidValue;        // at most 7 surplus workgroups, which return at once

    SlabArgs sl{};
    unsigned char *base = static_cast<unsigned char *>(ws);
    sl.state = single ? nullptr : reinterpret_cast<float *>(base);
    sl.tiles_cap = tpc * slab_chunks;
    sl.kimg = reinterpret_cast<uint16_t *>(base + state);
    sl.vimg = sl.kimg + (size_t)a.H * sl.tiles_cap * kImgElems;
    sl.tpc = (int)tpc;
    for (int64_t c0 = 0; c0 < a.n_chunks; c0 += slab_chunks) {
        const int64_t c1 = (c0 + slab_chunks < a.n_chunks) ? c0 + slab_chunks : a.n_chunks;
        // tiles of chunks c0 .. c1-1: tpc each, fewer in the cache's last chunk when it is short
        const int64_t last_len = ((c1 * a.chunk_len < a.n_kv) ? c1 * a.chunk_len : a.n_kv) - (c1 - 1) * a.chunk_len;
        sl.c0 = (int)c0;
        sl.n_tiles = (int)((c1 - 1 - c0) * tpc + (last_len + kAtKv - 1) / kAtKv);
        sl.first = c0 == 0;
        sl.last = c1 == a.n_chunks;
        if ((e = launch_slab_decode(a, sl, s)) != hipSuccess) return e;
        if (a.q_len) hipLaunchKernelGGL(attn_slab_kernel<true>, dim3((unsigned)(bpx * 8)), dim3(kAtThreads), kAtSmem, s, a, sl, (int)nqb, (int)nb, bpx);
        else hipLaunchKernelGGL(attn_slab_kernel<false>, dim3((unsigned)(bpx * 8)), dim3(kAtThreads), kAtSmem, s, a, sl, (int)nqb, (int)nb, bpx);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace qvg
