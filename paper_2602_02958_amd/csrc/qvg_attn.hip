// Attention that reads the compressed cache directly: O = softmax(scale * Q K_hat^T) V_hat,
// where K_hat / V_hat are the decoded values of paper Sec. 4.2 Eq. 7, rounded to bf16 as the
// stand-alone decoder stores them.  The decoded tiles live only in LDS.
//
// One workgroup = 8 wavefronts = 256 queries of one unit (32 per wavefront); it walks the cache
// chunk by chunk (each chunk has its own centroid tables) in tiles of 64 tokens.  Per tile:
//   1. S^T = K_tile . Q^T on v_mfma_f32_32x32x16_bf16: rows = cache tokens, columns = queries,
//      so a lane owns one query and the soft-max statistics stay in the lane (one exchange
//      between the two lane halves per tile);
//   2. online soft-max in fp32 (base-2 exponent);
//   3. O^T += V_tile^T . P on v_mfma_f32_32x32x16_f16: the probabilities go in as f16 (11
//      significant bits, round to nearest; bf16's 8 would cost up to 2^-9 of |V| in the output), and the V tile,
//      first rounded to bf16 like the stand-alone decoder's output, is stored as f16, which
//      holds every bf16 value of magnitude 2^-14 .. 65504 exactly (larger ones saturate).
//      The lane's P values are already the B operand: the V tile is stored transposed with
//      the matching token permutation, so no cross-lane traffic is needed;
//   4. all 512 threads decode the NEXT tile (2 tokens x 8 channels of K and of V each) into the
//      other LDS buffer, from data that was requested one or two tiles earlier.
// The decode work is amortised over 256 queries; only the two contractions use the matrix
// cores, the unpack / fma / soft-max work is VALU and is what bounds the kernel.
// Two kernels: attn_kernel_staged (one smoothing stage; 1..4 rounds of 2-bit levels with binary16
// or E4M3 scales, or one round of 4-bit levels with E4M3 scales; chunks that start on 16-byte
// boundaries of the scale array: the measured path) and attn_kernel_direct (everything else: more
// rounds, several smoothing stages, the other 4-bit forms).
// Both can rotate the decoded keys by a caller-supplied (cos, sin) table (keys are cached before
// the rotary embedding, Sec. 5 "Implementation") and read a prefix of caches allocated for more
// tokens.  A small third kernel merges two partial results by their log-sum-exps.
#include "qvg_attn_tiles.hpp"

namespace qvg {

// General variant: every thread loads its codes, scales and centroid rows straight from global
// memory (many small loads).  Used for more than 4 quantization rounds (their staging area would
// not fit in LDS), for chunks whose scale records do not start on 16-byte boundaries, and for
// several smoothing stages (the rows of all stages are added as they arrive).

template <int T_, int SM, int FMT, bool ROPE, bool QL>   // T_ > 0: compile-time stage count; 0: run-time (up to kMaxStages).
                                // SM: smoothing stages (a.S tables and id bytes): 1, 2..4, or 0 = a.S
                                // QL: a prefix length per query (a.q_len)
                                // FMT: stored format (kFmt* bits)
                                // ROPE: rotate the decoded keys by a.rope
__global__ __launch_bounds__(kAtThreads, 2)
void attn_kernel_direct(AttnArgs a, int n_qblocks, int n_blocks, int blocks_per_xcd) {
    constexpr int TM = T_ > 0 ? T_ : kMaxStages;
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t *Kt = reinterpret_cast<uint16_t *>(smem);                  // [2][64][136] bf16
    uint16_t *Vt = Kt + 2 * kKtElems;                                   // [2][128][72] f16, transposed

    // Workgroups are dealt to the 8 XCDs round-robin by their linear id; they are re-numbered so
    // that the query blocks of one unit run on one XCD and its cache is fetched into one L2 only
    // (as in the staged kernel below; the grid is padded to a multiple of 8)
    const int w = (int)(blockIdx.x % 8u) * blocks_per_xcd + (int)(blockIdx.x / 8u);
    if (w >= n_blocks) return;                                          // uniform, before any barrier
    const int h = w / n_qblocks;
    const int qblock = w - h * n_qblocks;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int64_t qrow = (int64_t)qblock * kAtQPerBlock + wave * 32 + col;
    const bool qvalid = qrow < a.n_q;
    // Prefix length per query (chunk-causal order for the queries of several chunks): the lane's
    // query sees tokens 0 .. qlen-1; wmin = the shortest prefix in the wavefront (tiles below it
    // need no mask); the workgroup walks the cache only up to its longest prefix.
    int qlen = 0x7fffffff, wmin = 0x7fffffff;
    Span sp = span_of(a);
    if (QL) {
        __shared__ int bmax;
        if (tid == 0) bmax = 1;
        __syncthreads();
        const int nk = (int)a.n_kv;
        int mx = 1;
        if (qvalid) { const int v = a.q_len[qrow]; qlen = v < 0 ? 0 : (v > nk ? nk : v); mx = qlen > 1 ? qlen : 1; }
        wmin = qlen;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const int o = __shfl_xor(wmin, off, 64); wmin = o < wmin ? o : wmin;
            const int p = __shfl_xor(mx, off, 64); mx = p > mx ? p : mx;
        }
        if (lane == 0) atomicMax(&bmax, mx);
        __syncthreads();
        sp.n_kv = bmax;
        sp.n_chunks = (int)((sp.n_kv + sp.chunk_len - 1) / sp.chunk_len);
        wmin = __builtin_amdgcn_readfirstlane(wmin);
    }
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

    // decode mapping: 16 adjacent lanes cover the 16 channel chunks of a token pair (coalesced)
    const int c8 = tid & 15, tp = tid >> 4;            // tp 0..31: tokens 2*tp, 2*tp+1 of the tile
    const int g = (c8 * 8) / B;
    // position of the token pair in a transposed V row: token 16*st + 8*a + 4*hh + e sits at
    // 16*st + 8*hh + 4*a + e (the order in which a lane's soft-max values feed the PV MFMA);
    // the 16-byte group index of a row is XOR-ed with a key, 2 * (row / 32), to spread the banks of
    // these transposing 4-byte stores.  The key must not change inside the 32 consecutive rows
    // that half a wavefront reads with one ds_read_b128 (measured: with 144-byte rows such a read
    // takes 5.3 cycles of LDS time when the 32 lanes use the same key, 8.5 when lanes 16..31 use
    // another one and 12.6 with a key per 8 rows, although every 16 lanes hit 16 different
    // groups in all three cases)
    const int tok = 2 * tp;
    const int v_pos = 16 * (tok >> 4) + 8 * ((tok >> 2) & 1) + 4 * ((tok >> 3) & 1) + (tok & 3);
    const int v_off = ((v_pos >> 3) ^ ((c8 >> 2) * 2)) * 8 + (v_pos & 7);      // in f16 units; rows 8*c8 .. 8*c8+7 have key 2*(row/32)

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

    uint4 rp[2];                      // (cos, sin) of the tile held in rk (ROPE only)
    auto decode_to_lds = [&](const Raw<TM, SM> &rk, const Raw<TM, SM> &rv, int buf) {
        float accA[8], accB[8];
        dequant2x8<T_, TM, SM, FMT>(rk, T, accA, accB);
        if (ROPE) { rope_rotate8(accA, rp[0]); rope_rotate8(accB, rp[1]); }
        uint16_t *kt = Kt + buf * kKtElems;
        *reinterpret_cast<uint4 *>(kt + (tok + 0) * kKtPitch + c8 * 8) = pack_bf16x8(accA);
        *reinterpret_cast<uint4 *>(kt + (tok + 1) * kKtPitch + c8 * 8) = pack_bf16x8(accB);
        dequant2x8<T_, TM, SM, FMT>(rv, T, accA, accB);
        uint16_t *vt = Vt + buf * kVtElems + v_off;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
            // round to bf16 (the decoder's output), then to f16 (exact in range): channels e, e+1
            const uint32_t pa = pack_bf16x2(accA[e], accA[e + 1]);
            const uint32_t pb = pack_bf16x2(accB[e], accB[e + 1]);
            *reinterpret_cast<uint32_t *>(vt + (c8 * 8 + e) * kVtPitch) = pack_f16x2_rtz(bf16_lo(pa), bf16_lo(pb));
            *reinterpret_cast<uint32_t *>(vt + (c8 * 8 + e + 1) * kVtPitch) = pack_f16x2_rtz(bf16_hi(pa), bf16_hi(pb));
        }
    };

    // ---- prologue: tile 0 into buffer 0, raw data of tile 1 in flight -------------------
    Tile cur = first_tile(sp);
    Tile nxt = next_tile(sp, cur);
    Tile nn = nxt.valid ? next_tile(sp, nxt) : nxt;
    uint32_t idk[2], idv[2];
    Raw<TM, SM> rk, rv;
    load_ids(ks, cur, tp, S, a.id_wide, idk);
    load_ids(vs, cur, tp, S, a.id_wide, idv);
    load_raw<T_, TM, SM, FMT>(ks, cur, tp, c8, T, G, g, K, S, idk, rk);
    load_raw<T_, TM, SM, FMT>(vs, cur, tp, c8, T, G, g, K, S, idv, rv);
    if (ROPE) load_rope(a.rope, cur, tp, c8, rp);
    load_ids(ks, nxt, tp, S, a.id_wide, idk);
    load_ids(vs, nxt, tp, S, a.id_wide, idv);
    decode_to_lds(rk, rv, 0);
    __syncthreads();

    int buf = 0;
    while (true) {
        // raw data of the next tile (consumed at the end of this iteration), ids of the one after
        if (nxt.valid) {
            load_raw<T_, TM, SM, FMT>(ks, nxt, tp, c8, T, G, g, K, S, idk, rk);
            load_raw<T_, TM, SM, FMT>(vs, nxt, tp, c8, T, G, g, K, S, idv, rv);
            if (ROPE) load_rope(a.rope, nxt, tp, c8, rp);
            load_ids(ks, nn, tp, S, a.id_wide, idk);
            load_ids(vs, nn, tp, S, a.id_wide, idv);
        }
        const uint16_t *kt = Kt + buf * kKtElems;
        const uint16_t *vt = Vt + buf * kVtElems;

        // ---- S^T = K_tile . Q^T -------------------------------------------
        floatx16_t S[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) S[nb][r] = 0.0f;
        {
            // K fragments are read kKAhead contractions ahead of their use (with fewer in flight
            // every pair of contractions waited for a whole LDS round trip)
            constexpr int kKAhead = 4;
            const uint16_t *arow = kt + col * kKtPitch + half * 8;
            auto kfrag = [&](int i) {
                return *reinterpret_cast<const bf16x8_t *>(arow + (i >> 3) * 32 * kKtPitch + (i & 7) * 16);
            };
            bf16x8_t kf[16];
#pragma unroll
            for (int i = 0; i < kKAhead; ++i) kf[i] = kfrag(i);
            __builtin_amdgcn_sched_group_barrier(0x100, kKAhead, 0);     // the first LDS reads
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                S[i >> 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    kf[i], __builtin_bit_cast(bf16x8_t, qa[i & 7]), S[i >> 3], 0, 0, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);       // one contraction
                if (i + kKAhead < 16) {
                    kf[i + kKAhead] = kfrag(i + kKAhead);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
                }
            }
        }
        // ---- online soft-max (base 2) --------------------------------------
        const int ntile = (int)((cur.cend - cur.t0 < kAtKv) ? cur.cend - cur.t0 : kAtKv);
        if (ntile < kAtKv) {                                   // uniform: last tile of a chunk
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kv = nb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                    if (kv >= ntile) S[nb][r] = -INFINITY;
                }
        }
        if (QL && cur.t0 + kAtKv > wmin) {                     // uniform: some query of the wavefront ends in or before this tile
            const int left = qlen - cur.t0;                    // tokens of this tile the lane's query sees (may be <= 0)
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
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64)) * scale2;     // the scale is positive: order kept
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
            for (int e = 0; e < 8; ++e)
                p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(S[st >> 1][(st & 1) * 8 + e], scale2, -m));
            pb[st] = make_uint4(pack_f16x2_rne(p[0], p[1]), pack_f16x2_rne(p[2], p[3]),
                                pack_f16x2_rne(p[4], p[5]), pack_f16x2_rne(p[6], p[7]));
            // the normaliser is the sum of the f16 probabilities the PV contraction uses, so that
            // numerator and denominator carry the same rounding
            l = sum_f16_pairs(pb[st], l);
        }
        // ---- O^T += V_tile^T . P --------------------------------------------
        {
            constexpr int kVAhead = 4;                            // V fragments in flight, as for K above
            auto vfrag = [&](int i) {
                const int mb = i >> 2, st = i & 3;
                const int key = mb * 2;                           // swizzle key of rows 32*mb .. 32*mb + 31
                return *reinterpret_cast<const halfx8_t *>(
                    vt + (mb * 32 + col) * kVtPitch + (((2 * st + half) ^ key) * 8));
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
        if (!nxt.valid) break;
        // ---- decode the next tile into the other buffer ------------------------
        decode_to_lds(rk, rv, buf ^ 1);
        __syncthreads();
        buf ^= 1;
        cur = nxt; nxt = nn;
        nn = nn.valid ? next_tile(sp, nn) : nn;
    }
    // ---- normalise and store: lane holds channels 32*mb + 8*g + 4*half + 0..3 of its query ----
    store_result(a, h, qrow, qvalid && (!QL || qlen > 0), qvalid, half, O, m, l);
}


// ---------------------------------------------------------------------------------------------
// Main variant (one smoothing stage, 1..4 rounds).  The packed codes and scales of a tile are
// brought in with a few wide loads per thread two tiles ahead and parked in an LDS staging
// area; the per-thread 2-byte reads that the decode needs then hit LDS instead of issuing
// dozens of tiny global loads.  The ids run three tiles ahead (a small ring in LDS), so that the
// centroid rows, the only per-thread gathers from global memory (L2), are requested a whole
// tile before they are used.
// ---------------------------------------------------------------------------------------------
constexpr int kStMaxT = 4;
constexpr int kStMaxG = 8;
constexpr int kStCodes = kAtKv * kStMaxT * 32;            // bytes of one side's codes of a tile
constexpr int kStScales = kAtKv * kStMaxT * kStMaxG * 2;  // bytes of one side's scales
constexpr int kStBytes = 2 * kStCodes + 2 * kStScales;   // K and V: codes, scales
constexpr size_t kAtSmemStaged = (size_t)2 * (kKtElems + kVtElems) * sizeof(uint16_t) + 2 * kStBytes + 4 * 2 * kAtKv;
constexpr size_t kAtSmemStagedWide = kAtSmemStaged + 4 * 2 * kAtKv;      // the id ring holds 16-bit words

template <bool V> struct BoolC { static constexpr bool value = V; };

template <int T_, bool ROPE, bool FP8, bool I4, bool WIDE, bool QL>   // ROPE: rotate the decoded keys by a.rope; FP8: E4M3 scale bytes;
                                                  // I4: 4-bit levels (64 code bytes per token and round, T_ <= 2);
                                                  // WIDE: 16-bit ids (more than 256 centroids);
                                                  // QL: a prefix length per query (a.q_len)
__global__ __launch_bounds__(kAtThreads, 2)
void attn_kernel_staged(AttnArgs a, int n_qblocks, int n_blocks, int blocks_per_xcd) {
    constexpr int T = T_;
    constexpr int CB = I4 ? 64 : 32;                                    // code bytes per token and round
    static_assert(kAtKv * T * CB <= kStCodes, "the codes of a tile must fit their staging area");
    extern __shared__ __align__(16) unsigned char smem[];
    uint16_t *Kt = reinterpret_cast<uint16_t *>(smem);                  // [2][64][136] bf16
    uint16_t *Vt = Kt + 2 * kKtElems;                                   // [2][128][72] f16, transposed
    unsigned char *stage = reinterpret_cast<unsigned char *>(Vt + 2 * kVtElems);   // [2][kStBytes]
    typedef typename std::conditional<WIDE, uint16_t, unsigned char>::type id_t;
    id_t *idring = reinterpret_cast<id_t *>(stage + 2 * kStBytes);      // [4][2][64]: ids run one tile further ahead

    // Workgroups are dealt to the 8 XCDs round-robin by their linear id; re-number them so that
    // the query blocks of one unit run on one XCD (two at a boundary) and the unit's compressed
    // cache is fetched into that XCD's L2 only, not into all eight.
    const int w = (int)(blockIdx.x % 8u) * blocks_per_xcd + (int)(blockIdx.x / 8u);
    if (w >= n_blocks) return;                                          // uniform, before any barrier
    const int h = w / n_qblocks;
    const int qblock = w - h * n_qblocks;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);          // uniform: lets whole waves branch
    const int col = lane & 31, half = lane >> 5;
    const int64_t qrow = (int64_t)qblock * kAtQPerBlock + wave * 32 + col;
    const bool qvalid = qrow < a.n_q;
    const int B = a.B, K = a.K;
    const int G = kHeadDim / B;
    const uint32_t kmax = (uint32_t)K - 1u;

    const id_t *k_ids = reinterpret_cast<const id_t *>(a.k_ids) + (int64_t)h * a.kv_stride;
    const id_t *v_ids = reinterpret_cast<const id_t *>(a.v_ids) + (int64_t)h * a.kv_stride;
    const uint8_t *k_codes = a.k_codes + (int64_t)h * a.kv_stride * T * CB, *v_codes = a.v_codes + (int64_t)h * a.kv_stride * T * CB;
    constexpr int SZ = FP8 ? 1 : 2;                                     // bytes of a stored scale
    const unsigned char *k_scales = reinterpret_cast<const unsigned char *>(a.k_scales) + (int64_t)h * a.kv_stride * T * G * SZ;
    const unsigned char *v_scales = reinterpret_cast<const unsigned char *>(a.v_scales) + (int64_t)h * a.kv_stride * T * G * SZ;
    const bf16_t *k_cent = a.k_cent + (int64_t)h * a.chunk_stride * K * kHeadDim;
    const bf16_t *v_cent = a.v_cent + (int64_t)h * a.chunk_stride * K * kHeadDim;

    const int c8 = tid & 15, tp = tid >> 4;            // tp 0..31: tokens 2*tp, 2*tp+1 of the tile
    const int g = (c8 * 8) / B;
    const int tok = 2 * tp;
    const int v_pos = 16 * (tok >> 4) + 8 * ((tok >> 2) & 1) + 4 * ((tok >> 3) & 1) + (tok & 3);
    const int v_off = ((v_pos >> 3) ^ ((c8 >> 2) * 2)) * 8 + (v_pos & 7);      // in f16 units; rows 8*c8 .. 8*c8+7 have key 2*(row/32)

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

    // ---- staging: what a thread fetches for a tile ------------------------------------------
    // 16-byte pieces, both sides: codes (a token-stage record is 32 B, or 64 B with 4-bit levels,
    // always 16-byte aligned; piece p of a side belongs to token p / (T * CB / 16)) and scales (T*G*2 bytes per token, contiguous
    // over the tile; the host picks this kernel only when chunks start 16-byte aligned).
    // Every step below comes in two forms: FULL (the tile has all 64 tokens: no per-token
    // predicates at all, the common case) and the general one.
    constexpr int kTokPieces = T * CB / 16;                          // code pieces of one token
    constexpr int kPieces = 2 * kAtKv * kTokPieces;                  // code pieces, both sides
    // the code pieces are fetched and parked by the first half of the wavefronts only: those
    // decode first and otherwise wait for the others at the barrier of every tile
    constexpr int kFetchThreads = kAtThreads / 2;
    constexpr int kPiecesPerThread = (kPieces + kFetchThreads - 1) / kFetchThreads;
    const int scPiecesSide = kAtKv * T * G * SZ / 16;                // scale pieces per side (<= 256)
    const int scBytesTok = T * G * SZ;                               // even (the host sees to it)
    struct Fetch { uint4 code[kPiecesPerThread]; uint4 sc; uint32_t id; };

    auto fetch_tile = [&](auto full, const Tile &t, Fetch &f) {
        constexpr bool FULL = decltype(full)::value;
        const int nvalid = FULL ? kAtKv : (t.valid ? (int)((t.cend - t.t0 < kAtKv) ? t.cend - t.t0 : kAtKv) : 0);
#pragma unroll
        for (int i = 0; i < kPiecesPerThread; ++i) {
            const int p = tid + i * kFetchThreads;
            if (!FULL) f.code[i] = make_uint4(0u, 0u, 0u, 0u);
            if (tid < kFetchThreads && p < kPieces) {
                const bool vside = p >= kPieces / 2;
                const int ps = p - (vside ? kPieces / 2 : 0);
                if (FULL || ps / kTokPieces < nvalid)
                    f.code[i] = *reinterpret_cast<const uint4 *>((vside ? v_codes : k_codes) +
                                                                 ((int64_t)t.t0 * T * CB + (int64_t)ps * 16));
            }
        }
        if (!FULL) f.sc = make_uint4(0u, 0u, 0u, 0u);
        if (tid < 2 * scPiecesSide) {
            const bool vside = tid >= scPiecesSide;
            const int ps = tid - (vside ? scPiecesSide : 0);
            // a piece is fetched when its first byte belongs to an existing token; the bytes of
            // later, missing tokens it may drag along are never used (their rows are masked)
            // and still lie inside this unit's scale array, except in the unit's very last
            // piece, which is fetched only if it ends inside the array.  All pieces of a full
            // tile lie inside the tile's own 64 records.
            const int64_t first = (int64_t)t.t0 * scBytesTok + (int64_t)ps * 16;
            if (FULL || ((ps * 16) / scBytesTok < nvalid && first + 16 <= (int64_t)a.n_kv * scBytesTok))
                f.sc = *reinterpret_cast<const uint4 *>((vside ? v_scales : k_scales) + first);
            else if ((ps * 16) / scBytesTok < nvalid) {
                // tail of the unit's array: 2 bytes at a time
                uint32_t w4[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int b = 0; b < 8; ++b)
                    if (first + 2 * b + 2 <= (int64_t)a.n_kv * scBytesTok)
                        w4[b >> 1] |= (uint32_t)*reinterpret_cast<const uint16_t *>((vside ? v_scales : k_scales) + first + 2 * b)
                                      << (16 * (b & 1));
                f.sc = make_uint4(w4[0], w4[1], w4[2], w4[3]);
            }
        }
    };
    // ids run one tile further ahead than codes and scales (the centroid rows they select are
    // gathered a whole tile before they are needed); a token that does not exist gets id 0.
    // The fetch only issues the load (of token 0 for a token that does not exist, so that the
    // load needs no branch); the zeroing and the clamp to the table's last row come with the
    // store: done at the fetch they made the fetching wavefronts wait for the id, and with it
    // for every load issued before it
    auto ids_valid = [&](const Tile &t) {
        return t.valid ? (int)((t.cend - t.t0 < kAtKv) ? t.cend - t.t0 : kAtKv) : 0;
    };
    auto fetch_ids = [&](const Tile &t, Fetch &f) {
        if (tid < 2 * kAtKv) {
            const int n = tid & 63;
            f.id = (uint32_t)((tid >> 6) ? v_ids : k_ids)[n < ids_valid(t) ? t.t0 + n : 0];
        }
    };
    auto park_ids = [&](const Tile &t, const Fetch &f, int ordinal) {
        if (tid < 2 * kAtKv)
            idring[(ordinal & 3) * 2 * kAtKv + tid] = (id_t)(((tid & 63) < ids_valid(t)) ? min(f.id, kmax) : 0u);
    };
    auto park_tile = [&](const Fetch &f, int sb) {
        unsigned char *st = stage + sb * kStBytes;
#pragma unroll
        for (int i = 0; i < kPiecesPerThread; ++i) {
            const int p = tid + i * kFetchThreads;
            if (tid < kFetchThreads && p < kPieces) {
                const bool vside = p >= kPieces / 2;
                const int ps = p - (vside ? kPieces / 2 : 0);
                *reinterpret_cast<uint4 *>(st + (vside ? kStCodes : 0) + ps * 16) = f.code[i];
            }
        }
        if (tid < 2 * scPiecesSide) {
            const bool vside = tid >= scPiecesSide;
            const int ps = tid - (vside ? scPiecesSide : 0);
            *reinterpret_cast<uint4 *>(st + 2 * kStCodes + (vside ? kStScales : 0) + ps * 16) = f.sc;
        }
    };
    // centroid rows of this thread's two tokens, both sides, using the parked ids (the id of a
    // token that does not exist is parked as 0)
    uint4 rp[2];                      // ROPE: (cos, sin) pairs of the tile whose rows are in cen
    auto gather_rows = [&](const Tile &t, int ordinal, uint4 cen[2][2]) {
        if (ROPE) load_rope(a.rope, t, tp, c8, rp);
        const id_t *st = idring + (ordinal & 3) * 2 * kAtKv;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const bf16_t *cent = (s ? v_cent : k_cent) + (int64_t)t.chunk * K * kHeadDim + c8 * 8;
#pragma unroll
            for (int e = 0; e < 2; ++e)
                cen[s][e] = *reinterpret_cast<const uint4 *>(cent + (int)st[s * kAtKv + tok + e] * kHeadDim);
        }
    };
    // decode the tile parked in staging buffer sb (rows gathered in cen) into tile buffer buf;
    // tokens that do not exist have zero codes and scales, and their rows are masked in the
    // soft-max, so whatever centroid row was gathered for them is harmless for K; V is zeroed
    auto decode_to_lds = [&](auto full, const Tile &t, int sb, const uint4 cen[2][2], int buf) {
        constexpr bool FULL = decltype(full)::value;
        const unsigned char *st = stage + sb * kStBytes;
        const int nvalid = FULL ? kAtKv : (int)((t.cend - t.t0 < kAtKv) ? t.cend - t.t0 : kAtKv);
        Raw<T> rs[2];                      // both sides are read before either is decoded
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            typedef typename std::conditional<I4, uint32_t, uint16_t>::type code_t;   // a thread's 8 channels of a round
            const code_t *cp = reinterpret_cast<const code_t *>(st + s * kStCodes) + tok * T * 16 + c8;
            typedef typename std::conditional<FP8, uint8_t, uint16_t>::type scale_t;
            const scale_t *sp = reinterpret_cast<const scale_t *>(st + 2 * kStCodes + s * kStScales) + tok * T * G + g;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
#pragma unroll
                for (int k = 0; k < T; ++k) {
                    rs[s].code[e][k] = cp[(e * T + k) * 16];
                    rs[s].sc[e][k] = sp[(e * T + k) * G];
                }
                rs[s].cen[e] = (FULL || tok + e < nvalid) ? cen[s][e] : make_uint4(0u, 0u, 0u, 0u);
            }
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const Raw<T> &r = rs[s];
            float accA[8], accB[8];
            dequant2x8<T, T, 1, (FP8 ? kFmtE4M3 : 0) | (I4 ? kFmtInt4 : 0)>(r, T, accA, accB);
            if (s == 0) {
                if (ROPE) { rope_rotate8(accA, rp[0]); rope_rotate8(accB, rp[1]); }
                uint16_t *kt = Kt + buf * kKtElems;
                *reinterpret_cast<uint4 *>(kt + (tok + 0) * kKtPitch + c8 * 8) = pack_bf16x8(accA);
                *reinterpret_cast<uint4 *>(kt + (tok + 1) * kKtPitch + c8 * 8) = pack_bf16x8(accB);
            } else {
                uint16_t *vt = Vt + buf * kVtElems + v_off;
#pragma unroll
                for (int e = 0; e < 8; e += 2) {
                    const uint32_t pa = pack_bf16x2(accA[e], accA[e + 1]);
                    const uint32_t pb2 = pack_bf16x2(accB[e], accB[e + 1]);
                    *reinterpret_cast<uint32_t *>(vt + (c8 * 8 + e) * kVtPitch) = pack_f16x2_rtz(bf16_lo(pa), bf16_lo(pb2));
                    *reinterpret_cast<uint32_t *>(vt + (c8 * 8 + e + 1) * kVtPitch) = pack_f16x2_rtz(bf16_hi(pa), bf16_hi(pb2));
                }
            }
        }
    };
    auto is_full = [&](const Tile &t) { return t.valid && t.cend - t.t0 >= kAtKv; };

    // ---- prologue: tile 0 decoded into buffer 0, tile 1 parked, ids of tiles 0..2 parked ------
    // QL: the lane's query sees tokens 0 .. qlen-1; wmin = the shortest prefix in the wavefront
    // (tiles below it need no mask); the workgroup walks the cache up to its longest prefix only
    int qlen = 0x7fffffff, wmin = 0x7fffffff;
    Span sp = span_of(a);
    if (QL) {
        __shared__ int bmax;
        if (tid == 0) bmax = 1;
        __syncthreads();
        const int nk = (int)a.n_kv;
        int mx = 1;
        if (qvalid) { const int v = a.q_len[qrow]; qlen = v < 0 ? 0 : (v > nk ? nk : v); mx = qlen > 1 ? qlen : 1; }
        wmin = qlen;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const int o = __shfl_xor(wmin, off, 64); wmin = o < wmin ? o : wmin;
            const int p = __shfl_xor(mx, off, 64); mx = p > mx ? p : mx;
        }
        if (lane == 0) atomicMax(&bmax, mx);
        __syncthreads();
        sp.n_kv = bmax;
        sp.n_chunks = (int)((sp.n_kv + sp.chunk_len - 1) / sp.chunk_len);
        wmin = __builtin_amdgcn_readfirstlane(wmin);
    }
    Tile cur = first_tile(sp);
    Tile nxt = next_tile(sp, cur);
    Tile nn = nxt.valid ? next_tile(sp, nxt) : nxt;
    Tile n3 = nn.valid ? next_tile(sp, nn) : nn;
    Fetch f;
    uint4 cen[2][2];
    fetch_tile(BoolC<false>{}, cur, f);  fetch_ids(cur, f);  park_tile(f, 0);  park_ids(cur, f, 0);
    fetch_tile(BoolC<false>{}, nxt, f);  fetch_ids(nxt, f);  park_tile(f, 1);  park_ids(nxt, f, 1);
    fetch_ids(nn, f);  park_ids(nn, f, 2);
    __syncthreads();
    gather_rows(cur, 0, cen);
    decode_to_lds(BoolC<false>{}, cur, 0, cen, 0);
    if (nxt.valid) gather_rows(nxt, 1, cen);
    __syncthreads();                 // tile 0 ready; staging buffer 0 free again

    int buf = 0;                     // tile buffer of `cur`; the staging buffer of `nxt` is buf ^ 1
    int jt = 0;                      // ordinal of `cur`
    // S, soft-max and PV on `cur`
    auto compute = [&](auto full) {
        constexpr bool FULL = decltype(full)::value;
        const uint16_t *kt = Kt + buf * kKtElems;
        const uint16_t *vt = Vt + buf * kVtElems;
        floatx16_t S[2];
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) S[nb][r] = 0.0f;
        {
            // the sixteen K fragments are read kKAhead contractions ahead of their use: with
            // fewer in flight every pair of contractions waited for a whole LDS round trip
            constexpr int kKAhead = 4;
            const uint16_t *arow = kt + col * kKtPitch + half * 8;
            auto kfrag = [&](int i) {
                return *reinterpret_cast<const bf16x8_t *>(arow + (i >> 3) * 32 * kKtPitch + (i & 7) * 16);
            };
            bf16x8_t kf[16];
#pragma unroll
            for (int i = 0; i < kKAhead; ++i) kf[i] = kfrag(i);
            __builtin_amdgcn_sched_group_barrier(0x100, kKAhead, 0);     // the first LDS reads
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                S[i >> 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    kf[i], __builtin_bit_cast(bf16x8_t, qa[i & 7]), S[i >> 3], 0, 0, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);       // one contraction
                if (i + kKAhead < 16) {
                    kf[i + kKAhead] = kfrag(i + kKAhead);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
                }
            }
        }
        if (!FULL) {
            const int ntile = (int)((cur.cend - cur.t0 < kAtKv) ? cur.cend - cur.t0 : kAtKv);
            if (ntile < kAtKv) {                                   // uniform: last tile of a chunk
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int kv = nb * 32 + (r >> 2) * 8 + half * 4 + (r & 3);
                        if (kv >= ntile) S[nb][r] = -INFINITY;
                    }
            }
        }
        if (QL && cur.t0 + kAtKv > wmin) {                     // uniform: some query of the wavefront ends in or before this tile
            const int left = qlen - cur.t0;                    // tokens of this tile the lane's query sees (may be <= 0)
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
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64)) * scale2;     // the scale is positive: order kept
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
            for (int e = 0; e < 8; ++e)
                p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(S[st >> 1][(st & 1) * 8 + e], scale2, -m));
            pb[st] = make_uint4(pack_f16x2_rne(p[0], p[1]), pack_f16x2_rne(p[2], p[3]),
                                pack_f16x2_rne(p[4], p[5]), pack_f16x2_rne(p[6], p[7]));
            // the normaliser is the sum of the f16 probabilities the PV contraction uses, so that
            // numerator and denominator carry the same rounding
            l = sum_f16_pairs(pb[st], l);
        }
        {
            constexpr int kVAhead = 4;                            // V fragments in flight, as for K above
            auto vfrag = [&](int i) {
                const int mb = i >> 2, st = i & 3;
                const int key = mb * 2;                           // swizzle key of rows 32*mb .. 32*mb + 31
                return *reinterpret_cast<const halfx8_t *>(
                    vt + (mb * 32 + col) * kVtPitch + (((2 * st + half) ^ key) * 8));
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
    };
    // One tile of the main loop.  Two independent parts: compute on `cur`, and decode of `nxt`
    // into the other tile buffer (its raw data was parked before the previous barrier, its rows
    // were gathered an iteration ago) followed by the gather for `nn`.  Half of the wavefronts
    // run the parts in the opposite order (decode_first), so that on every SIMD one wavefront is
    // in a matrix-core phase while the other is in a VALU phase.  Codes and scales of `nn` and
    // ids of `n3` are fetched at the top and parked at the bottom.  FULL: cur, nxt and nn all
    // hold 64 tokens.  Returns false after the last tile.
    auto tile_step = [&](auto full, bool decode_first /* uniform; only honoured with FULL */) -> bool {
        constexpr bool FULL = decltype(full)::value;
        // codes and scales of `nn` and ids of `n3` land during this iteration; a wavefront that
        // decodes first issues them after the decode, whose waits for the gathered rows would
        // otherwise (the load counter is in order) also wait for these fresh loads
        if (FULL && decode_first) {
            decode_to_lds(full, nxt, buf ^ 1, cen, buf ^ 1);
            gather_rows(nn, jt + 2, cen);
            fetch_tile(full, nn, f);
            fetch_ids(n3, f);
        } else {
            if (FULL || nn.valid) fetch_tile(full, nn, f);
            fetch_ids(n3, f);
        }
        compute(full);
        if (!FULL && !nxt.valid) return false;
        if (!(FULL && decode_first)) {
            decode_to_lds(full, nxt, buf ^ 1, cen, buf ^ 1);
            if (FULL || nn.valid) gather_rows(nn, jt + 2, cen);
        }
        if (FULL || nn.valid) park_tile(f, buf);                   // staging buf is free since the last barrier
        park_ids(n3, f, jt + 3);
        __syncthreads();
        buf ^= 1;
        jt += 1;
        cur = nxt; nxt = nn; nn = n3;
        n3 = n3.valid ? next_tile(sp, n3) : n3;
        return true;
    };
    // wavefronts w and w + 4 share a SIMD: the first four decode first (measured: 3 % over all
    // wavefronts in the same order; matrix-core and VALU work of two wavefronts overlap only little)
    const bool decode_first = wave < kAtWaves / 2;
    while (true) {
        while (is_full(cur) && is_full(nxt) && is_full(nn)) tile_step(BoolC<true>{}, decode_first);
        if (!tile_step(BoolC<false>{}, false)) break;
    }
    store_result(a, h, qrow, qvalid && (!QL || qlen > 0), qvalid, half, O, m, l);
}

template <int T_, bool ROPE, bool FP8, bool I4, bool WIDE, bool QL = false>
static hipError_t launch_attn_staged_r(const AttnArgs &a, hipStream_t s) {
    constexpr size_t kSmem = WIDE ? kAtSmemStagedWide : kAtSmemStaged;
    static LdsHighWater lds_limit = {};
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(&attn_kernel_staged<T_, ROPE, FP8, I4, WIDE, QL>), kSmem, lds_limit);
    if (e != hipSuccess) return e;
    const int64_t nqb = (a.n_q + kAtQPerBlock - 1) / kAtQPerBlock;
    const int64_t nb = nqb * a.H;
    if (nb > 0x7fffffff - 8) return hipErrorInvalidValue;
    const int bpx = (int)((nb + 7) / 8);
    // the grid is padded to a multiple of 8 (one share per XCD): at most 7 surplus workgroups, whose
    // renumbered index is >= nb; each returns on its first statement, before it forms a unit index
    if ((int64_t)bpx * 8 > nb + 7) return hipErrorInvalidValue;
    hipLaunchKernelGGL((attn_kernel_staged<T_, ROPE, FP8, I4, WIDE, QL>), dim3((unsigned)(bpx * 8)), dim3(kAtThreads), kSmem, s, a,
                       (int)nqb, (int)nb, bpx);
    return hipGetLastError();
}
template <int T_, bool FP8 = false, bool I4 = false, bool WIDE = false>
static hipError_t launch_attn_staged(const AttnArgs &a, hipStream_t s) {
    return a.rope ? launch_attn_staged_r<T_, true, FP8, I4, WIDE>(a, s) : launch_attn_staged_r<T_, false, FP8, I4, WIDE>(a, s);
}

template <int T_, int SM, int FMT, bool ROPE, bool QL = false>
static hipError_t launch_attn_tr(const AttnArgs &a, hipStream_t s) {
    static LdsHighWater lds_limit = {};
    hipError_t e = ensure_dynamic_lds(reinterpret_cast<const void *>(&attn_kernel_direct<T_, SM, FMT, ROPE, QL>), kAtSmem, lds_limit);
    if (e != hipSuccess) return e;
    const int64_t nqb = (a.n_q + kAtQPerBlock - 1) / kAtQPerBlock;
    const int64_t nb = nqb * a.H;
    if (nb > 0x7fffffff - 8) return hipErrorInvalidValue;
    const int bpx = (int)((nb + 7) / 8);
    if ((int64_t)bpx * 8 > nb + 7) return hipErrorInvalidValue;        // at most 7 surplus workgroups, which return at once
    hipLaunchKernelGGL((attn_kernel_direct<T_, SM, FMT, ROPE, QL>), dim3((unsigned)(bpx * 8)), dim3(kAtThreads), kAtSmem, s, a,
                       (int)nqb, (int)nb, bpx);
    return hipGetLastError();
}
template <int T_, int SM, int FMT = 0>
static hipError_t launch_attn_t(const AttnArgs &a, hipStream_t s) {
    return a.rope ? launch_attn_tr<T_, SM, FMT, true>(a, s) : launch_attn_tr<T_, SM, FMT, false>(a, s);
}
// several smoothing stages: the paper's form (two or four stages, one round) with the stage count
// fixed at compile time, anything else with run-time counts
template <int FMT>
static hipError_t launch_attn_multi(const AttnArgs &a, hipStream_t s) {
    // (16-bit ids with several stages: the run-time-count instances, which read the ids stage by stage)
    if (a.T == 1 && a.S == 4 && !a.id_wide) return launch_attn_t<1, 4, FMT>(a, s);
    if (a.T == 1 && a.S == 2 && !a.id_wide) return launch_attn_t<1, 2, FMT>(a, s);
    return a.T == 1 ? launch_attn_t<1, 0, FMT>(a, s) : launch_attn_t<0, 0, FMT>(a, s);
}

// the other stored formats run on the general kernel
template <int FMT>
static hipError_t launch_attn_fmt(const AttnArgs &a, hipStream_t s) {
    if (a.S > 1) return launch_attn_multi<FMT>(a, s);
    if (a.T == 1) return launch_attn_t<1, 1, FMT>(a, s);       // the paper's single round
    return launch_attn_t<0, 1, FMT>(a, s);
}

template <int FMT>
static hipError_t launch_attn_qlen(const AttnArgs &a, hipStream_t s) {
    if (a.S > 1) return a.rope ? launch_attn_tr<0, 0, FMT, true, true>(a, s) : launch_attn_tr<0, 0, FMT, false, true>(a, s);
    return a.rope ? launch_attn_tr<0, 1, FMT, true, true>(a, s) : launch_attn_tr<0, 1, FMT, false, true>(a, s);
}

template <int T_>
static hipError_t launch_attn_staged_qlen(const AttnArgs &a, hipStream_t s) {
    return a.rope ? launch_attn_staged_r<T_, true, false, false, false, true>(a, s)
                  : launch_attn_staged_r<T_, false, false, false, false, true>(a, s);
}

hipError_t launch_attn(const AttnArgs &a, hipStream_t s) {
    if (a.n_q == 0) return hipSuccess;
    if (a.q_len) {
        // a prefix per query: the staged kernel for the plain format (2-bit levels, binary16 scales,
        // one smoothing stage, byte ids, up to 4 rounds, aligned chunks); else instances of the
        // general kernel with run-time counts
        const bool al = ((a.chunk_len % 8 == 0) || a.n_chunks == 1) &&
            (reinterpret_cast<uintptr_t>(a.k_scales) & 15u) == 0 && (reinterpret_cast<uintptr_t>(a.v_scales) & 15u) == 0 &&
            (a.H == 1 || (a.kv_stride * a.T * (kHeadDim / a.B) * 2) % 16 == 0);
        if (a.fmt == 0 && a.S == 1 && !a.id_wide && al && a.T <= kStMaxT) {
            switch (a.T) {
                case 1: return launch_attn_staged_qlen<1>(a, s);
                case 2: return launch_attn_staged_qlen<2>(a, s);
                case 3: return launch_attn_staged_qlen<3>(a, s);
                default: return launch_attn_staged_qlen<4>(a, s);
            }
        }
        switch (a.fmt) {
            case 0: return launch_attn_qlen<0>(a, s);
            case kFmtE4M3: return launch_attn_qlen<kFmtE4M3>(a, s);
            case kFmtInt4: return launch_attn_qlen<kFmtInt4>(a, s);
            default: return launch_attn_qlen<kFmtInt4 | kFmtE4M3>(a, s);
        }
    }
    // the staged kernel fetches scales in 16-byte pieces: every chunk must start on one
    // (binary16 scales: chunk_len * T * G * 2 bytes a multiple of 16; the test below is the sufficient
    // chunk_len % 8 == 0) and so must every unit's array (units are kv_stride tokens apart)
    const bool aligned = ((a.chunk_len % 8 == 0) || a.n_chunks == 1) &&
        (reinterpret_cast<uintptr_t>(a.k_scales) & 15u) == 0 && (reinterpret_cast<uintptr_t>(a.v_scales) & 15u) == 0 &&
        (a.H == 1 || (a.kv_stride * a.T * (kHeadDim / a.B) * ((a.fmt & kFmtE4M3) ? 1 : 2)) % 16 == 0);
    // E4M3 scales on the staged kernel: a token's scale record must have an even number of bytes
    // (the tail handling moves two at a time) and every unit's scale array must start on a
    // 16-byte boundary
    const bool fp8_staged_any = a.S == 1 && aligned && ((a.T * (kHeadDim / a.B)) & 1) == 0 &&
        ((reinterpret_cast<uintptr_t>(a.k_scales) | reinterpret_cast<uintptr_t>(a.v_scales)) & 15u) == 0 &&
        (a.H == 1 || (a.kv_stride * a.T * (kHeadDim / a.B)) % 16 == 0);
    if (a.id_wide) {
        // 16-bit ids (more than 256 centroids): the form of the paper's codebook-size study (2-bit
        // levels, E4M3 scales, one round) has a staged instance, everything else runs on the general kernel
        if (a.fmt == kFmtE4M3 && fp8_staged_any && a.T == 1) return launch_attn_staged<1, true, false, true>(a, s);
        switch (a.fmt) {
            case 0: return a.S > 1 ? launch_attn_multi<0>(a, s) : launch_attn_t<0, 1>(a, s);
            case kFmtE4M3: return launch_attn_fmt<kFmtE4M3>(a, s);
            case kFmtInt4: return launch_attn_fmt<kFmtInt4>(a, s);
            default: return launch_attn_fmt<kFmtInt4 | kFmtE4M3>(a, s);
        }
    }
    const bool fp8_staged = fp8_staged_any;
    switch (a.fmt) {
        case 0: break;
        case kFmtE4M3:
            // 2-bit levels with E4M3 scales (the paper's own format)
            if (fp8_staged && a.T <= kStMaxT) {
                switch (a.T) {
                    case 1: return launch_attn_staged<1, true>(a, s);
                    case 2: return launch_attn_staged<2, true>(a, s);
                    case 3: return launch_attn_staged<3, true>(a, s);
                    default: return launch_attn_staged<4, true>(a, s);
                }
            }
            return launch_attn_fmt<kFmtE4M3>(a, s);
        case kFmtInt4: return launch_attn_fmt<kFmtInt4>(a, s);
        default:
            // 4-bit levels with E4M3 scales, one round (the paper's INT4 format)
            if (fp8_staged && a.T == 1) return launch_attn_staged<1, true, true>(a, s);
            return launch_attn_fmt<kFmtInt4 | kFmtE4M3>(a, s);
    }
    // several smoothing stages: the general kernel (the paper's presets have one round)
    if (a.S > 1) return launch_attn_multi<0>(a, s);
    if (!aligned || a.T > kStMaxT) return launch_attn_t<0, 1>(a, s);
    switch (a.T) {
        case 1: return launch_attn_staged<1>(a, s);
        case 2: return launch_attn_staged<2>(a, s);
        case 3: return launch_attn_staged<3>(a, s);
        default: return launch_attn_staged<4>(a, s);
    }
}

// ---------------------------------------------------------------------------------------------
// Merge of two partial attention results over disjoint key sets (the compressed cache and the
// current chunk's own keys) into the attention over their union, from the outputs and the
// log-sum-exps: w_a = exp(lse_a - m), w_b = exp(lse_b - m), m = max; o = (w_a o_a + w_b o_b) /
// (w_a + w_b); lse = m + log(w_a + w_b).  16 lanes per row, 8 channels each: a streaming pass.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256)
void attn_merge_kernel(MergeArgs a) {
    const int64_t r = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4);
    const int c8 = threadIdx.x & 15;
    if (r >= a.rows) return;
    const float la = a.lsea[r], lb = a.lseb[r];
    const float m = fmaxf(la, lb);
    const float wa = __builtin_amdgcn_exp2f((la - m) * 1.4426950408889634f);
    const float wb = __builtin_amdgcn_exp2f((lb - m) * 1.4426950408889634f);
    const float z = wa + wb, inv = 1.0f / z;
    float xa[8], xb[8], o[8];
    unpack_bf16x8(*reinterpret_cast<const uint4 *>(a.oa + r * kHeadDim + c8 * 8), xa);
    unpack_bf16x8(*reinterpret_cast<const uint4 *>(a.ob + r * kHeadDim + c8 * 8), xb);
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (wa * xa[i] + wb * xb[i]) * inv;
    *reinterpret_cast<uint4 *>(a.out + r * kHeadDim + c8 * 8) = pack_bf16x8(o);
    if (a.lse && c8 == 0) a.lse[r] = m + __builtin_log2f(z) * 0.6931471805599453f;
}

hipError_t launch_attn_merge(const MergeArgs &a, hipStream_t s) {
    if (a.rows == 0) return hipSuccess;
    const int64_t nb = (a.rows + 15) / 16;
    if (nb > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attn_merge_kernel, dim3((unsigned)nb), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace qvg
