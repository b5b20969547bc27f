// Prefill attention (chunks of any length over the cache, then the append) and the
// soft-gated attention forward, on gfx950: keys staged in the page layout, tiles shared by a
// workgroup through LDS, MFMA tile loop with lazily raised softmax references.
#include "spkv_device.h"

// ------------------------------------------------- prefill attention (any chunk length)
// n new tokens per sequence attend causally with the availability rule of Eq. 3-4 and are
// appended, in four steps:
//   1. spkv_prefill_stage copies the window as it stands (ring, un-rotated into position
//      order) and the n new K/V rows into staging half-pages in the page layout: staging
//      row u holds position T_old - w + u, so query i (position T_old + i) has exactly the
//      rows i < u <= i + w in its window.
//   2. the bulk append runs and records, per new token, how long a prefix of the long-term
//      list lies at least w behind it (see spkv_bulk_ring).
//   3. spkv_prefill_attend: one wave per block of tb = 32 / G consecutive tokens of one
//      (sequence, KV head) -- 32 MFMA columns (token, head) in two groups of 16; one group
//      for the shortest chunks -- walks the long-term prefix and then the staging rows of
//      the block's windows, one online softmax per column, and writes the normalised bf16
//      rows (or, when a span's keys are cut into ranges, partial results that
//      spkv_prefill_combine merges).
// Window keys and long-term entries are disjoint (positions > t - w against <= t - w), so
// every available key is counted once.

struct SpkvPrefill {
    uint16_t* stage;     // [n_pairs][shp] half-pages
    int32_t*  prefix;    // [total tokens][H_kv]
    float*    bias;      // soft gating only: [n_pairs][shp][32] log2 u of every staging row
    int32_t   shp;       // staging half-pages per pair
    int32_t   tb;        // tokens per wave (16 nq / G)
    int32_t   nblk;      // workgroups (spans of nw tb tokens) per pair in the grid
    int32_t   pin_xcd;   // 1: all blocks of a pair run on one XCD (shared L2)
    int32_t   nw;        // waves per workgroup (2, 4 or 8): a span is nw * tb tokens
    int32_t   nq;        // column groups of 16 per wave (1 or 2)
    int32_t   ks;        // workgroups per span: the span's tiles are cut into ks ranges (split-K)
    float*    part;      // ks > 1: partial (acc, m, l) of every (span, range, column)
};

// One workgroup per (staging half-page, pair): wave wv fills rows 8 wv .. 8 wv + 7.  Rows
// without a position (before the sequence start, past the chunk) are zero, so that a
// masked key never meets a non-finite V element.  Runs BEFORE the append (reads the ring
// and the token count as they were).
// With pf.bias set (soft gating) it also stores log2 u = log2 sigmoid(f) of every new row.
template <int D>
__global__ __launch_bounds__(256) void spkv_prefill_stage(SpkvView v, const uint16_t* __restrict__ k,
                                                          const uint16_t* __restrict__ vv,
                                                          const float* __restrict__ f, SpkvCu cu,
                                                          SpkvPrefill pf) {
    const int pair = blockIdx.y, sh = blockIdx.x;
    const int b = pair / v.Hkv, h = pair - b * v.Hkv;
    const int row0 = cu.v[b], n = cu.v[b + 1] - row0;
    if (n == 0 || sh * kHalfTokens >= v.w + n) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, c = lane & 15;
    const int T0 = v.t_pair[pair];
    __shared__ __attribute__((aligned(16))) uint16_t s_v[4][8][D];
    uint16_t* dp = pf.stage + ((size_t)pair * pf.shp + sh) * (size_t)(2 * kHalfTokens * D);
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        const int row = pass * 4 + (lane >> 4);
        const int u = sh * kHalfTokens + wave * 8 + row;
        if (c < D / 8) {
            uint4 kk = {0u, 0u, 0u, 0u}, vl = {0u, 0u, 0u, 0u};
            if (u >= v.w) {
                const int j = u - v.w;
                if (j < n) {
                    const size_t src = ((size_t)(row0 + j) * v.Hkv + h) * D + c * 8;
                    kk = *reinterpret_cast<const uint4*>(k + src);
                    vl = *reinterpret_cast<const uint4*>(vv + src);
                }
            } else {
                const int s = T0 - v.w + u;
                if (s >= 0) {
                    const int slot = s % v.w;
                    const uint16_t* sp = ring_page(v, pair, slot >> 6);
                    const int sk = slot & 63;
                    kk = *reinterpret_cast<const uint4*>(sp + spkv_k_off(D, sk, c * 8));
                    const uint16_t* vs = sp + spkv_v_off(D, sk, c * 8);
                    unsigned wd[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        wd[e] = (unsigned)vs[(2 * e) * 8] | ((unsigned)vs[(2 * e + 1) * 8] << 16);
                    vl = make_uint4(wd[0], wd[1], wd[2], wd[3]);
                }
            }
            *reinterpret_cast<uint4*>(dp + spkv_k_off(D, wave * 8 + row, c * 8)) = kk;
            *reinterpret_cast<uint4*>(&s_v[wave][row][c * 8]) = vl;
        }
        if (pf.bias != nullptr && c == 0) {
            float lb = 0.f;
            if (u >= v.w && u - v.w < n) {
                // log u = log sigmoid(f) = -softplus(-f) (Eq. 1 and the soft gate), in log2
                const float x = f[((size_t)row0 + (u - v.w)) * v.Hkv + h];
                const float ls = x < -20.f ? x : -log1pf(__expf(-x));
                lb = ls * 1.4426950408889634f;
            }
            pf.bias[((size_t)pair * pf.shp + sh) * kHalfTokens + wave * 8 + row] = lb;
        }
    }
    __builtin_amdgcn_wave_barrier();
    store_v_units<D>(dp, wave * 8, s_v[wave], lane);
}

// Bits e = 0..7 set for a <= e <= b (empty if the range misses 0..7); branch-free.
__device__ __forceinline__ unsigned bit_range8(int a, int b) {
    const int lo = min(max(a, 0), 8), hi = max(min(b, 7), -8);
    return (0xffu << lo) & (0xffu >> (7 - hi)) & 0xffu;
}

// One half-page from LDS for the NQ column groups of a wave, in pieces so that the
// accumulators are only ever touched by MFMA inside the tile loop:
//   tile_scores      S = K Q^T for the groups (2 NQ independent accumulator chains),
//                    masked keys to -inf
//   tile_weights     weights p = 2^(x - m) against the column references m as they stand,
//                    and their per-lane sums; reports (wave-uniform) whether a reference
//                    is too low -- some sum above 2^11, so a weight may exceed 2^8 -- or
//                    not set yet.  Weights up to 2^11 are harmless in bf16 / fp32, so in
//                    the steady state no maximum is taken and nothing is rescaled.
//   tile_accumulate  sums and P V with the weights accepted
//   rescale_columns  raises the references to the column maxima of the tile and rescales
//                    sums and accumulators; the tile loop leaves its inner loop for this
//                    (rare once a few tiles have been seen) and then redoes the tile
constexpr float kWeightSumLimit = 2048.0f;
// Shape of a workgroup: long chunks take eight waves of two column groups of 16 (two waves
// per SIMD, one workgroup per compute unit, 256 query columns per tile fetch).  Chunks of
// fewer tokens than eight such waves hold would leave waves without a token, so they get
// four waves of two groups, and the shortest four or two waves of one group each (measured
// on 16-token chunks: as fast as two waves of two groups on 16 sequences at 32k, 10 % faster
// on 4 sequences at 128k; eight waves of one group for 32 tokens were 15 % slower than four
// of two -- twice the waves read every tile from LDS).
static SpkvPrefillShape prefill_shape(int group, int n_max) {
    SpkvPrefillShape sh;
    const int tb1 = 16 / group, tb2 = 32 / group;    // tokens of one, two column groups (group <= 16)
    if (n_max <= 4 * tb1) {
        sh.nq = 1;
        sh.nw = n_max <= 2 * tb1 ? 2 : 4;
    } else {
        sh.nq = 2;
        sh.nw = n_max <= 4 * tb2 ? 4 : 8;
    }
    sh.tb = 16 * sh.nq / group;
    return sh;
}

template <int D, int NQ>
__device__ __forceinline__ void tile_scores(const uint16_t* tile, int lane,
                                            const bf16x8 (&qb)[NQ][D / 32], const unsigned (&kill)[NQ],
                                            bool any_kill, float (&x)[NQ][8]) {
    constexpr int NS = D / 32;
    f32x4 s0[NQ], s1[NQ];
#pragma unroll
    for (int c = 0; c < NQ; ++c) {
        s0[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
        s1[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int sl = 0; sl < NS; ++sl) {
        const bf16x8 k0 = *reinterpret_cast<const bf16x8*>(tile + sl * 512 + lane * 8);
        const bf16x8 k1 = *reinterpret_cast<const bf16x8*>(tile + (NS + sl) * 512 + lane * 8);
#pragma unroll
        for (int c = 0; c < NQ; ++c) {
            s0[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, qb[c][sl], s0[c], 0, 0, 0);
            s1[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, qb[c][sl], s1[c], 0, 0, 0);
        }
    }
#pragma unroll
    for (int c = 0; c < NQ; ++c) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[c][i] = s0[c][i];
            x[c][4 + i] = s1[c][i];
        }
    }
    if (any_kill) {
#pragma unroll
        for (int c = 0; c < NQ; ++c)
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if ((kill[c] >> e) & 1u) x[c][e] = SPKV_NEG_INF;
    }
}

template <int NQ>
__device__ __forceinline__ bool tile_weights(const float (&x)[NQ][8], float scale_log2e,
                                             const float (&m)[NQ], f32x8 (&p)[NQ], float (&psum)[NQ]) {
    bool low = false;
#pragma unroll
    for (int c = 0; c < NQ; ++c) {
        const bool unset = m[c] == SPKV_NEG_INF;
        const float neg_ref = unset ? 0.f : -m[c];
        float sum = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            p[c][e] = __builtin_amdgcn_exp2f(__builtin_fmaf(x[c][e], scale_log2e, neg_ref));
            sum += p[c][e];
        }
        psum[c] = sum;
        low = low || unset || !(sum <= kWeightSumLimit);
    }
    return __ballot(low) != 0ull;
}

template <int D, int NQ>
__device__ __forceinline__ void tile_accumulate(const uint16_t* tile, int lane, const f32x8 (&p)[NQ],
                                                const float (&psum)[NQ], f32x4 (&acc)[NQ][D / 16],
                                                float (&l)[NQ]) {
    constexpr int NS = D / 32, NB = D / 16;
    bf16x8 va[NB];
#pragma unroll
    for (int db = 0; db < NB; ++db)
        va[db] = *reinterpret_cast<const bf16x8*>(tile + (2 * NS + db) * 512 + lane * 8);
#pragma unroll
    for (int c = 0; c < NQ; ++c) {
        l[c] += psum[c];
        const bf16x8 pb = __builtin_convertvector(p[c], bf16x8);
#pragma unroll
        for (int db = 0; db < NB; ++db)
            acc[c][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[db], pb, acc[c][db], 0, 0, 0);
    }
}

// x: the masked scores of the tile that did not fit the references.  A column whose keys
// are all excluded so far keeps the reference -inf (its sums and accumulators are zero).
template <int D, int NQ>
__device__ __forceinline__ void rescale_columns(const float (&x)[NQ][8], float scale_log2e,
                                                f32x4 (&acc)[NQ][D / 16], float (&m)[NQ], float (&l)[NQ]) {
#pragma unroll
    for (int c = 0; c < NQ; ++c) {
        float cm = fmaxf(fmaxf(fmaxf(x[c][0], x[c][1]), fmaxf(x[c][2], x[c][3])),
                         fmaxf(fmaxf(x[c][4], x[c][5]), fmaxf(x[c][6], x[c][7]))) * scale_log2e;
        cm = fmaxf(cm, __shfl_xor(cm, 16));
        cm = fmaxf(cm, __shfl_xor(cm, 32));
        const float m_new = fmaxf(m[c], cm);
        const float m_ref = (m_new == SPKV_NEG_INF) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m[c] - m_ref);
        l[c] *= alpha;
#pragma unroll
        for (int db = 0; db < D / 16; ++db) acc[c][db] *= alpha;
        m[c] = m_new;
    }
}

// One workgroup of NW (8, for short chunks 4 or 2) waves per span of NW * tb consecutive tokens of one
// (sequence, KV head); wave wv owns tokens i0 = span start + wv * tb .. + tb - 1 as its
// 16 NQ MFMA columns (tb = 16 NQ / G tokens times G heads; NQ = 2 groups of 16, one for the
// shortest chunks).  The waves walk the
// same half-pages, so each 16 KB tile is fetched from memory once per workgroup into a ring
// of LDS buffers (every wave copies its share of a tile straight from memory into LDS, two
// tiles ahead of the one all waves consume) and each wave reads its MFMA A operands from LDS
// with conflict-free 16-byte reads; 256 query columns share one tile fetch.  With 32 columns a wave needs about 200 VGPRs and
// no accumulation registers, so two waves fit a SIMD and one wave's vector work (weights)
// can run beside the other's MFMAs.  (Measured alternatives: four waves of 64 columns, one
// per SIMD, 15 % slower -- every latency is exposed; the same with the tile loop software-
// pipelined by hand, slower still; issue priority for one wave of each SIMD, 27 % slower.)
template <int D, bool SOFT, int NW, int NQ>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2, 2))) void spkv_prefill_attend(SpkvView v, const uint16_t* __restrict__ q,
                                                           uint16_t* __restrict__ out,
                                                           float* __restrict__ lse, float scale_log2e,
                                                           SpkvPrefill pf, SpkvCu cu) {
    constexpr int NS = D / 32, NB = D / 16;
    constexpr int kHalfElems = 2 * kHalfTokens * D;
    constexpr int kRows = kHalfElems / 512;     // 1 KB rows of a tile
    constexpr int kRowsPerWave = kRows / NW;
    // Tiles in flight ahead of the one in use (three measured no faster than two, for long
    // chunks and for the two-wave workgroups of short ones alike).
    constexpr int kAhead = 2, kBufs = kAhead + 1;
    __shared__ __attribute__((aligned(16))) uint16_t s_tile[kBufs][kHalfElems];
    int pair, qblk, kr;      // (sequence, KV head), span, tile range of the span
    if (pf.pin_xcd) {
        // workgroups go round-robin to the 8 XCDs: id % 8 picks the XCD, and every pair
        // lives on XCD pair % 8, so its list is fetched into one L2 and re-read there
        const int local = blockIdx.x >> 3, lp = local / (pf.nblk * pf.ks);
        const int rem = local - lp * pf.nblk * pf.ks;
        qblk = rem / pf.ks;
        kr = rem - qblk * pf.ks;
        // rotate inside every full group of 8 pairs by the group index: with 8 KV heads a
        // plain pair % 8 would give each XCD one head of every sequence, and heads differ
        // several-fold in kept length
        const int rot = (lp * 8 + 8 <= v.n_pairs) ? lp : 0;
        pair = lp * 8 + (((blockIdx.x & 7) + rot) & 7);
        if (pair >= v.n_pairs) return;
    } else {
        pair = blockIdx.x / (pf.nblk * pf.ks);
        const int rem = blockIdx.x - pair * pf.nblk * pf.ks;
        qblk = rem / pf.ks;
        kr = rem - qblk * pf.ks;
    }
    qblk = pf.nblk - 1 - qblk;            // longest prefixes first
    const int b = pair / v.Hkv, h = pair - b * v.Hkv;
    const int row0 = cu.v[b], n_tok = cu.v[b + 1] - row0;
    const int span0 = qblk * NW * pf.tb;
    if (span0 >= n_tok) return;
    const int span_last = min(span0 + NW * pf.tb, n_tok) - 1;
    const int tid = threadIdx.x, lane = tid & 63, kc = lane >> 4, n = lane & 15;
    // wave index as a scalar: everything derived from it (token range, loop bounds, the
    // branches on them) then stays in scalar registers and scalar branches
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int i0 = span0 + wv * pf.tb;
    const int tbv = max(0, min(pf.tb, n_tok - i0)), i_last = i0 + tbv - 1, cols = tbv * v.G;
    const bool active = tbv > 0;
    // the cache is in the state after the append
    const int T0 = SOFT ? 0 : v.t_pair[pair] - n_tok, L = SOFT ? 0 : v.kept_len[pair];
    const int u_min = max(0, v.w - T0);     // first staging row that holds a position

    auto prefix_of = [&](int i) -> int {   // long-term entries at least w behind token i
        if (SOFT || T0 + i - v.w < 0) return 0;
        return min(max(pf.prefix[((size_t)row0 + i) * v.Hkv + h], 0), L);
    };

    bf16x8 qb[NQ][NS];
    int tok[NQ], cnt[NQ];
#pragma unroll
    for (int c = 0; c < NQ; ++c) {
        const int col = c * 16 + n;
        const int i = i0 + col / v.G, g = col - (col / v.G) * v.G;
        const bool valid = col < cols;
        tok[c] = valid ? i : -1;
        cnt[c] = valid ? prefix_of(i) : 0;
        const uint16_t* qrow = q + ((size_t)(row0 + i) * v.Hq + (size_t)h * v.G + g) * D + kc * 8;
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) {
            uint4 raw = {0u, 0u, 0u, 0u};
            if (valid) raw = *reinterpret_cast<const uint4*>(qrow + sl * 32);
            qb[c][sl] = __builtin_bit_cast(bf16x8, raw);
        }
    }
    // long-term half-pages: the workgroup visits those some token of the span can see; this
    // wave computes on those below its own last count, unmasked below its first count
    const int nA = (prefix_of(span_last) + kHalfTokens - 1) >> 5;
    const int nA_wave = active ? (prefix_of(i_last) + kHalfTokens - 1) >> 5 : 0;
    const int fullA = active ? prefix_of(i0) >> 5 : 0;
    // staging half-pages: rows (span0, span_last + w] that hold a position; this wave's
    // windows cover rows [lo_w, hi_w]
    const int sB0 = (SOFT ? u_min : max(span0 + 1, u_min)) >> 5;
    const int nB = ((span_last + v.w) >> 5) - sB0 + 1;
    const int lo_w = SOFT ? u_min : max(i0 + 1, u_min), hi_w = i_last + v.w;
    const int n_hp = nA + nB, last = n_hp - 1;
    // split-K: this workgroup takes tiles [x_begin, x_end) of the span's n_hp
    const int x_begin = (int)(((long long)kr * n_hp) / pf.ks);
    const int x_end = (int)(((long long)(kr + 1) * n_hp) / pf.ks);

    const int32_t* pt = v.page_table + (size_t)pair * v.pt_cap;
    const uint16_t* stage = pf.stage + (size_t)pair * pf.shp * (size_t)kHalfElems;
    // Page ids are fetched 64 at a time, one per lane, and picked by readlane: the tile
    // loop then issues no memory load of its own whose wait would also wait for the tile
    // copies in flight (a fetch happens once per 128 tiles and is waited for on the spot).
    int page_lane0 = -64, my_page = 0;      // logical page held by lane 0; this lane's page id
    auto page_of = [&](int lp) -> int {     // lp wave-uniform, never decreasing
        if (lp >= page_lane0 + 64) {
            page_lane0 = lp;
            my_page = pt[min(lp + lane, v.pt_cap - 1)];
            __builtin_amdgcn_s_waitcnt(0x0f70);          // vmcnt(0)
        }
        return __builtin_amdgcn_readlane(my_page, lp - page_lane0);
    };
    auto base_of = [&](int x) -> const uint16_t* {
        x = min(x, last);
        if (x < nA) {
            const int page = min(max(page_of(min(x >> 1, v.pt_cap - 1)), 0), v.n_pages - 1);
            return pool_page(v, page) + (x & 1) * kHalfElems;
        }
        return stage + (size_t)min(sB0 + x - nA, pf.shp - 1) * kHalfElems;
    };

    f32x4 acc[NQ][NB];
    float m[NQ], l[NQ];
#pragma unroll
    for (int c = 0; c < NQ; ++c) {
        m[c] = SPKV_NEG_INF;
        l[c] = 0.f;
#pragma unroll
        for (int i = 0; i < NB; ++i) acc[c][i] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }

    // Tiles go from memory straight into LDS (no registers in between), two tiles ahead of
    // their use: the copy of tile x + 2 is issued when tile x is begun, into the buffer that
    // tile x - 1 vacated, and has a whole tile's time more than it needs before the barrier
    // that ends tile x + 1's wait.  Every wave copies its kRowsPerWave 1 KB rows of a tile;
    // a wave-wide 16-byte load lands at the row's LDS address plus 16 bytes per lane.
    const int my_off = (wv * kRowsPerWave * 64 + lane) * 8;     // this lane's part of a tile
    const unsigned lds_rows = (unsigned)(uintptr_t)(__attribute__((address_space(3))) uint16_t*)&s_tile[0][0] +
                              (unsigned)wv * (kRowsPerWave * 1024);
    // Soft gating: the 32 biases log2 u of a tile's rows travel the same way, every wave
    // fetching a copy of its own (lanes 32-63 repeat lanes 0-31), so that the tile loop
    // issues no load whose wait would also wait for the copies in flight.
    __shared__ __attribute__((aligned(16))) float s_bias[SOFT ? kBufs : 1][SOFT ? NW : 1][SOFT ? 64 : 4];
    const unsigned lds_bias = (unsigned)(uintptr_t)(__attribute__((address_space(3))) float*)&s_bias[0][0][0] +
                              (unsigned)wv * 256;
    constexpr int kCopiesPerTile = kRowsPerWave + (SOFT ? 1 : 0);   // loads a wave issues per tile
    auto stage_tile = [&](const uint16_t* base, int xt, int buf) {    // tile xt (for the biases)
        const uint16_t* p = base + my_off;
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r)
            load_row_to_lds(p + r * 512, lds_rows + (unsigned)buf * (kHalfElems * 2) + r * 1024);
        if (SOFT) {
            const int hp = min(sB0 + min(xt, last) - nA, pf.shp - 1);
            load_word_to_lds(pf.bias + ((size_t)pair * pf.shp + hp) * kHalfTokens + (lane & 31),
                             lds_bias + (unsigned)buf * (NW * 256));
        }
    };
    // Everything loaded so far (queries, counts) is waited for here, once: left pending, the
    // first use inside the tile loop would carry a wait for all loads in flight -- on every
    // tile, tile copies included.
    __builtin_amdgcn_s_waitcnt(0x0f70);          // vmcnt(0)
    stage_tile(base_of(x_begin), x_begin, 0);
#pragma unroll
    for (int a = 1; a < kAhead; ++a) stage_tile(base_of(x_begin + a), x_begin + a, a);
    const uint16_t* p_next = base_of(x_begin + kAhead);
    wait_loads_but<(kAhead - 1) * kCopiesPerTile>();        // tile x_begin has landed
    __syncthreads();

    // Tile loop.  The inner loop never touches the accumulators except by MFMA; when the
    // references do not fit a tile the wave leaves it before using the tile, rescales, and
    // resumes at the same tile (prefetch and barrier of a tile are issued exactly once, so
    // the waves stay in step whatever each one does).  After a rescale the references
    // are at least the tile's column maxima, so the second attempt is accepted; a column
    // with every key excluded so far keeps m = -inf and is accepted on the retry as well.
    int x = x_begin, buf = 0;            // buf: LDS buffer of tile x
    bool resume = false, pending = false;
    float xs[NQ][8];
    while (x < x_end) {
        if (pending) rescale_columns<D, NQ>(xs, SOFT ? 1.0f : scale_log2e, acc, m, l);
        for (; x < x_end; ++x) {
            if (!resume) {
                // the tile after next (past the last one: the last tile again, never used)
                stage_tile(p_next, x + kAhead, buf >= 1 ? buf - 1 : kBufs - 1);
                p_next = base_of(x + kAhead + 1);
            }
            resume = false;
            const uint16_t* tile = s_tile[buf];
            bool mine;
            int u_tile = 0;
            if (x < nA) {
                mine = x < nA_wave;
            } else {
                u_tile = (sB0 + x - nA) * kHalfTokens;
                mine = active && u_tile <= hi_w && u_tile + kHalfTokens > lo_w;
            }
            if (mine) {
                // per column group: which of this lane's eight keys are excluded
                unsigned kill[NQ] = {};
                bool any = true;
                if (x < nA) {
                    any = x >= fullA;
                    if (any) {
                        const int k0 = x * kHalfTokens + kc * 8;   // list index of this lane's first key
#pragma unroll
                        for (int c = 0; c < NQ; ++c) kill[c] = bit_range8(0, cnt[c] - k0 - 1) ^ 0xffu;
                    }
                } else {
                    // soft gating: a tile of rows that all hold a position and all lie at or
                    // before every token of the wave needs no mask
                    if (SOFT && u_tile >= u_min && u_tile + kHalfTokens - 1 <= i0 + v.w) any = false;
                    const int u0 = u_tile + kc * 8;
                    // window of token i: rows i < u <= i + w that hold a position (soft
                    // gating: every earlier row as well)
#pragma unroll
                    for (int c = 0; c < NQ; ++c)
                        kill[c] = (tok[c] >= 0 ? bit_range8((SOFT ? u_min : max(tok[c] + 1, u_min)) - u0,
                                                            tok[c] + v.w - u0)
                                               : 0u) ^ 0xffu;
                }
                tile_scores<D, NQ>(tile, lane, qb, kill, any, xs);
                if (SOFT) {
                    // scores to the log2 domain plus the gate bias log2 u of every key outside
                    // the window of its query (row u <= i); masked scores stay -inf
                    const int u0 = u_tile + kc * 8;
                    const float4* bp = reinterpret_cast<const float4*>(&s_bias[SOFT ? buf : 0][SOFT ? wv : 0][SOFT ? kc * 8 : 0]);
                    const float4 b0 = bp[0], b1 = bp[1];
                    const float bias[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
                    if (u_tile + kHalfTokens - 1 <= i0) {       // outside every window of the wave
#pragma unroll
                        for (int c = 0; c < NQ; ++c)
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                xs[c][e] = __builtin_fmaf(xs[c][e], scale_log2e, bias[e]);
                    } else {
#pragma unroll
                        for (int c = 0; c < NQ; ++c)
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                xs[c][e] = __builtin_fmaf(xs[c][e], scale_log2e,
                                                          u0 + e <= tok[c] ? bias[e] : 0.f);
                    }
                }
                f32x8 pw[NQ];
                float psum[NQ];
                if (tile_weights<NQ>(xs, SOFT ? 1.0f : scale_log2e, m, pw, psum) && !pending) {
                    pending = true;
                    resume = true;
                    break;
                }
                pending = false;
                tile_accumulate<D, NQ>(tile, lane, pw, psum, acc, l);
            }
            wait_loads_but<(kAhead - 1) * kCopiesPerTile>();    // all but the newest copies: tile x + 1 has landed
            __syncthreads();
            buf = buf == kBufs - 1 ? 0 : buf + 1;
        }
    }
    wait_loads_but<0>();

#pragma unroll
    for (int c = 0; c < NQ; ++c) {
        float lc = l[c];
        lc += __shfl_xor(lc, 16);
        lc += __shfl_xor(lc, 32);
        if (tok[c] >= 0 && pf.ks > 1) {
            // partial of this tile range: un-normalised accumulators, reference, sum
            // layout: [all columns][D] accumulators, then [all columns][2] (m, l)
            const size_t n_cols = (size_t)v.n_pairs * pf.nblk * pf.ks * (NW * NQ * 16);
            const size_t pc = (((size_t)pair * pf.nblk + qblk) * pf.ks + kr) * (NW * NQ * 16) +
                              wv * (NQ * 16) + c * 16 + n;
            float* pa = pf.part + pc * D + kc * 4;
#pragma unroll
            for (int db = 0; db < NB; ++db) *reinterpret_cast<f32x4*>(pa + db * 16) = acc[c][db];
            if (kc == 0) {
                pf.part[n_cols * D + pc * 2] = m[c];
                pf.part[n_cols * D + pc * 2 + 1] = lc;
            }
        } else if (tok[c] >= 0) {
            const int col = c * 16 + n;
            const int g = col - (col / v.G) * v.G;
            const size_t o = (size_t)(row0 + tok[c]) * v.Hq + (size_t)h * v.G + g;
            const float inv = 1.0f / lc;
            uint16_t* po = out + o * D + kc * 4;
#pragma unroll
            for (int db = 0; db < NB; ++db) {
                const __bf16 r0 = (__bf16)(acc[c][db][0] * inv), r1 = (__bf16)(acc[c][db][1] * inv);
                const __bf16 r2 = (__bf16)(acc[c][db][2] * inv), r3 = (__bf16)(acc[c][db][3] * inv);
                uint2 pk;
                pk.x = (unsigned)__builtin_bit_cast(uint16_t, r0) | ((unsigned)__builtin_bit_cast(uint16_t, r1) << 16);
                pk.y = (unsigned)__builtin_bit_cast(uint16_t, r2) | ((unsigned)__builtin_bit_cast(uint16_t, r3) << 16);
                *reinterpret_cast<uint2*>(po + db * 16) = pk;
            }
            if (lse != nullptr && kc == 0) lse[o] = (m[c] + log2f(lc)) * 0.6931471805599453f;
        }
    }
}

// Merge of the tile ranges of one (span, column): out = sum_r 2^(m_r - M) acc_r /
// sum_r 2^(m_r - M) l_r.  A workgroup of 256 threads takes 256 / (D / 4) consecutive columns
// of a span's workgroup; a thread owns four consecutive output elements of one column.
template <int D>
__global__ __launch_bounds__(256) void spkv_prefill_combine(SpkvView v, uint16_t* __restrict__ out,
                                                            float* __restrict__ lse, SpkvPrefill pf,
                                                            SpkvCu cu) {
    constexpr int TPC = D / 4, CPB = 256 / TPC;          // threads per column, columns per block
    const int kCols = pf.nw * pf.nq * 16;               // a multiple of CPB (of 16)
    const int blocks_per_span = kCols / CPB;
    const int span = blockIdx.x / blocks_per_span;
    const int cs = (blockIdx.x - span * blocks_per_span) * CPB + (int)threadIdx.x / TPC;
    const int d = ((int)threadIdx.x % TPC) * 4;
    const int pair = span / pf.nblk, qblk = span - pair * pf.nblk;
    const int b = pair / v.Hkv, h = pair - b * v.Hkv;
    const int row0 = cu.v[b], n_tok = cu.v[b + 1] - row0;
    const int wv = cs / (pf.nq * 16), col = cs - wv * (pf.nq * 16);
    const int i0 = qblk * pf.nw * pf.tb + wv * pf.tb;
    const int tbv = max(0, min(pf.tb, n_tok - i0));
    if (col >= tbv * v.G) return;
    const int i = i0 + col / v.G, g = col - (col / v.G) * v.G;
    const size_t n_cols = (size_t)v.n_pairs * pf.nblk * pf.ks * kCols;
    const size_t pc0 = (size_t)span * pf.ks * kCols + cs;      // range r: pc0 + r * kCols
    const float* ml = pf.part + n_cols * D;
    float M = SPKV_NEG_INF;
    for (int r = 0; r < pf.ks; ++r) M = fmaxf(M, ml[(pc0 + (size_t)r * kCols) * 2]);
    f32x4 num = {0.f, 0.f, 0.f, 0.f};
    float den = 0.f;
    for (int r = 0; r < pf.ks; ++r) {
        const size_t pc = pc0 + (size_t)r * kCols;
        const float sc = __builtin_amdgcn_exp2f(ml[pc * 2] - M);      // 0 for a range without keys
        num += *reinterpret_cast<const f32x4*>(pf.part + pc * D + d) * sc;
        den += ml[pc * 2 + 1] * sc;
    }
    const size_t o = (size_t)(row0 + i) * v.Hq + (size_t)h * v.G + g;
    const float inv = 1.0f / den;
    uint2 packed;
    packed.x = (unsigned)__builtin_bit_cast(uint16_t, (__bf16)(num[0] * inv)) |
               ((unsigned)__builtin_bit_cast(uint16_t, (__bf16)(num[1] * inv)) << 16);
    packed.y = (unsigned)__builtin_bit_cast(uint16_t, (__bf16)(num[2] * inv)) |
               ((unsigned)__builtin_bit_cast(uint16_t, (__bf16)(num[3] * inv)) << 16);
    *reinterpret_cast<uint2*>(out + o * D + d) = packed;
    if (lse != nullptr && d == 0) lse[o] = (M + log2f(den)) * 0.6931471805599453f;
}

static SpkvPrefill prefill_params(const SpkvView& v, int n_max, uint16_t* stage, int32_t* prefix,
                                  float* bias, int shp, int ks = 1, float* part = nullptr) {
    SpkvPrefill pf;
    pf.ks = ks;
    pf.part = part;
    pf.stage = stage;
    pf.prefix = prefix;
    pf.bias = bias;
    pf.shp = shp;
    const SpkvPrefillShape sh = prefill_shape(v.G, n_max);
    pf.tb = sh.tb;
    pf.nw = sh.nw;
    pf.nq = sh.nq;
    pf.nblk = (n_max + pf.nw * pf.tb - 1) / (pf.nw * pf.tb);   // spans of one workgroup
    pf.pin_xcd = (v.n_pairs >= 8 && pf.nblk * pf.ks >= 4) ? 1 : 0;
    return pf;
}

static unsigned prefill_grid(const SpkvView& v, const SpkvPrefill& pf) {
    return pf.pin_xcd ? 8u * (unsigned)((v.n_pairs + 7) / 8) * (unsigned)(pf.nblk * pf.ks)
                      : (unsigned)v.n_pairs * (unsigned)(pf.nblk * pf.ks);
}

SpkvPrefillShape spkv_prefill_shape(int group, int n_max) { return prefill_shape(group, n_max); }

int spkv_prefill_spans(int n_pairs, int group, int n_max) {
    const SpkvPrefillShape sh = prefill_shape(group, n_max);
    return n_pairs * ((n_max + sh.nw * sh.tb - 1) / (sh.nw * sh.tb));
}

size_t spkv_prefill_partial_bytes(int spans, int ks, SpkvPrefillShape sh, int head_dim) {
    return ks > 1 ? (size_t)spans * ks * (sh.nw * sh.nq * 16) * (head_dim + 2) * 4 : 0;
}

// The attention launch of the shape chosen for the call.
template <int D, bool SOFT>
static void launch_attend(const SpkvView& v, const uint16_t* q, uint16_t* out, float* lse, float sl,
                          const SpkvPrefill& pf, const SpkvCu& cu, unsigned grid, hipStream_t s) {
    if (pf.nq == 2 && pf.nw == 8)
        spkv_prefill_attend<D, SOFT, 8, 2><<<dim3(grid), dim3(512), 0, s>>>(v, q, out, lse, sl, pf, cu);
    else if (pf.nq == 2)
        spkv_prefill_attend<D, SOFT, 4, 2><<<dim3(grid), dim3(256), 0, s>>>(v, q, out, lse, sl, pf, cu);
    else if (pf.nw == 4)
        spkv_prefill_attend<D, SOFT, 4, 1><<<dim3(grid), dim3(256), 0, s>>>(v, q, out, lse, sl, pf, cu);
    else
        spkv_prefill_attend<D, SOFT, 2, 1><<<dim3(grid), dim3(128), 0, s>>>(v, q, out, lse, sl, pf, cu);
}

hipError_t spkv_launch_prefill(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                               const float* f, const uint16_t* q, uint16_t* out, float* lse,
                               float sm_scale, const SpkvCu& cu, int n_max, uint16_t* stage,
                               int32_t* prefix, int shp, int ks, float* part, hipStream_t s) {
    const SpkvPrefill pf = prefill_params(v, n_max, stage, prefix, nullptr, shp, ks, part);
    const float sl = sm_scale * 1.4426950408889634f;
    const int stage_hps = (v.w + n_max + kHalfTokens - 1) / kHalfTokens;
    const unsigned grid = prefill_grid(v, pf);
    hipError_t e;
    if (v.D == 128) {
        spkv_prefill_stage<128><<<dim3(stage_hps, v.n_pairs), dim3(256), 0, s>>>(v, k, vv, f, cu, pf);
        if ((e = spkv_launch_append_bulk(v, k, vv, f, cu, n_max, prefix, s)) != hipSuccess) return e;
        launch_attend<128, false>(v, q, out, lse, sl, pf, cu, grid, s);
        if (ks > 1)
            spkv_prefill_combine<128><<<dim3(v.n_pairs * pf.nblk * pf.nw * pf.nq * 16 / 8), dim3(256), 0, s>>>(v, out, lse, pf, cu);
    } else {
        spkv_prefill_stage<64><<<dim3(stage_hps, v.n_pairs), dim3(256), 0, s>>>(v, k, vv, f, cu, pf);
        if ((e = spkv_launch_append_bulk(v, k, vv, f, cu, n_max, prefix, s)) != hipSuccess) return e;
        launch_attend<64, false>(v, q, out, lse, sl, pf, cu, grid, s);
        if (ks > 1)
            spkv_prefill_combine<64><<<dim3(v.n_pairs * pf.nblk * pf.nw * pf.nq * 16 / 16), dim3(256), 0, s>>>(v, out, lse, pf, cu);
    }
    return hipGetLastError();
}

// Soft-gated attention of whole sequences (no cache): the same staging and the same tile
// loop with every earlier row visible and the bias log2 u on the rows outside the window.
// v: a view that only describes the shape (B, heads, D, w, n_pairs) and whose t_pair points
// at n_pairs zeros.
hipError_t spkv_launch_soft_gated(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                                  const float* f, const uint16_t* q, uint16_t* out, float* lse,
                                  float sm_scale, const SpkvCu& cu, int n_max, uint16_t* stage,
                                  float* bias, int shp, hipStream_t s) {
    const SpkvPrefill pf = prefill_params(v, n_max, stage, nullptr, bias, shp);
    const float sl = sm_scale * 1.4426950408889634f;
    const int stage_hps = (v.w + n_max + kHalfTokens - 1) / kHalfTokens;
    const unsigned grid = prefill_grid(v, pf);
    if (v.D == 128) {
        spkv_prefill_stage<128><<<dim3(stage_hps, v.n_pairs), dim3(256), 0, s>>>(v, k, vv, f, cu, pf);
        launch_attend<128, true>(v, q, out, lse, sl, pf, cu, grid, s);
    } else {
        spkv_prefill_stage<64><<<dim3(stage_hps, v.n_pairs), dim3(256), 0, s>>>(v, k, vv, f, cu, pf);
        launch_attend<64, true>(v, q, out, lse, sl, pf, cu, grid, s);
    }
    return hipGetLastError();
}

