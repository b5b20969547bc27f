// Read path of the SP-KV cache on gfx950 (MI355X, wave64, MFMA):
//   spkv_decode_split    split-K flash decoding, one wave per work item, K/V tiles consumed
//                        as MFMA operands straight from the page layout
//   spkv_decode_combine  log-sum-exp merge of the partials
//   fused step           spkv_decode_split<.., true> + spkv_combine_append: append and decode
//                        of one token per sequence in two launches instead of three; with
//                        the utility predictor riding along: spkv_decode_split_predict
//   multi-token step     spkv_chunk_split + spkv_chunk_combine: up to 16 new tokens per sequence
#include "spkv_device.h"

// One wavefront per work item.  The G <= 16 query heads of the GQA group are the N = 16
// columns of every MFMA, so each K/V tile is read exactly once per group.  Every wave-wide
// load is 1 KB contiguous.
// MW = sp.mw consecutive items of a pair form a workgroup.  With MW > 1 the waves work
// independently and meet once, at the end, to merge their (max, sum, acc) triples in LDS, so
// that one partial per workgroup goes to memory (the partial stores sit in the tail of every
// wave; a quarter of them measured 1.5-2 us less per launch) and the merge launch has a
// quarter to fold.  The host picks MW > 1 only when packing the items of every pair into whole
// workgroups does not lengthen the items (few pairs with long lists).
// Block id = pair * slots + jj with an odd slot count: workgroups go round-robin to the 8
// XCDs, so the items of every pair -- long or short -- spread evenly over all of them
// (heads differ in kept length by several times; pinning a head to one XCD would leave
// the others idle), and the odd stride keeps the per-pair remainders from piling up on
// the low XCDs.
//
// FUSED = false: the cache already holds the newest token (spkv_append ran before).
// FUSED = true (spkv_decode_step): the cache is in the state before the append of the
// newest token.  The kernel then excludes the ring slot that token will overwrite unless
// the pair in it passes the gate (it is the pair leaving the window: kept -> it stays
// attended, as the next long-term entry; dropped -> it is gone), and publishes every
// pair's item count for spkv_combine_append, which adds the new token's own term.
//
// Modes of the split kernel:
//   kSplitPlain     partials only (spkv_decode_attention in two launches, split-only timing)
//   kSplitFusedTwo  first launch of the two-launch fused step (FUSED above)
//   kSplitMerge     one launch for spkv_decode_attention: every workgroup of a (sequence, KV
//                   head), with or without work, takes a ticket of the pair once its partial
//                   (stored through to device scope) has arrived; the one that draws the last
//                   ticket -- all partials of the pair are then visible to it after a
//                   device-scope acquire -- merges them and writes `out` / `lse`
//   kSplitStep      one launch for the whole fused step: kSplitMerge in the state before the
//                   append (FUSED masking), the merging workgroup adds the new token's own term
//                   and then performs the pair's append.  Workgroups without work take a
//                   ticket too because they have read the pair's counters: the append may only
//                   change them once nobody will read them again in this launch.
// No workgroup ever waits for another: tickets are a single fetch-and-add, so the launch
// drains whatever the order in which its workgroups run.
constexpr int kSplitPlain = 0, kSplitFusedTwo = 1, kSplitMerge = 2, kSplitStep = 3;
constexpr int kMergePad = 16;    // floats between the rows of the LDS copy: no bank conflicts for G = 4

static size_t split_lds_bytes(int mw, int group, int head_dim) {
    if (mw == 1) return 0;
    return ((size_t)mw * group * (head_dim + kMergePad) + 2 * mw * 16) * sizeof(float);
}

// The work of one workgroup that has some: MW items of pair `pair`, their partial to slot
// pair * slots + jj.
template <int D, bool FUSED, int MW, bool SHARED>
__device__ __forceinline__ void split_compute(const SpkvView& v, const uint16_t* __restrict__ q,
                                              float scale_log2e, SpkvSplit sp, const PairSplit& ps,
                                              int pair, int jj, float* s_mem) {
    constexpr int NS = D / 32;   // head-dim slabs of one K tile
    constexpr int NB = D / 16;   // 16-wide output blocks
    const int wave = MW == 1 ? 0 : __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int j = jj * MW + wave;
    // a wave past the pair's last item takes an empty range and joins the merge with weight 0
    const bool has_item = j < ps.items;
    const int hbase = ps.nhp / ps.items, hrem = ps.nhp - hbase * ps.items;
    const int hp0 = has_item ? j * hbase + min(j, hrem) : 0;
    const int hp1 = has_item ? hp0 + hbase + (j < hrem ? 1 : 0) : 0;
    const int b = pair / v.Hkv, h = pair - b * v.Hkv;
    const int lane = threadIdx.x & 63, kc = lane >> 4, n = lane & 15;

    bf16x8 qb[NS];
    {
        const uint16_t* qrow = q + ((size_t)b * v.Hq + (size_t)h * v.G + n) * D + kc * 8;
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) {
            uint4 raw = {0u, 0u, 0u, 0u};
            if (n < v.G) raw = *reinterpret_cast<const uint4*>(qrow + sl * 32);
            qb[sl] = __builtin_bit_cast(bf16x8, raw);
        }
    }
    f32x4 acc[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float m = SPKV_NEG_INF, l = 0.f;
    const int32_t* pt = v.page_table + (size_t)pair * v.pt_cap;

    // Fused step: which ring key (if any) must be left out.  Only items that reach into
    // the ring look (most do not), and only after their query loads are under way.
    int drop_hp = -1, drop_r = -1;
    if (FUSED && hp1 > ps.ghp && ps.T >= v.w) {
        const int slot = ps.T % v.w;
        if (!gate_passes(v, v.ring_logit[(size_t)pair * v.w + slot], ps.T - v.w)) {
            drop_hp = ps.ghp + (slot >> 5);
            drop_r = slot & 31;
        }
    }

    int hp = hp0;
    while (hp < hp1) {
        // Page ids of the next 64 logical pages, one per lane; read back with readlane so
        // that no half-page waits on a dependent table lookup.
        const int pbase = hp >> 1;
        const int my_page = pt[min(pbase + lane, v.pt_cap - 1)];
        const int hp_end = min(hp1, (pbase + 64) << 1);
        for (; hp < hp_end; ++hp) {
            const uint16_t* base;
            int nvalid;
            if (hp < ps.ghp) {
                const int page = __builtin_amdgcn_readlane(my_page, (hp >> 1) - pbase);
                base = pool_page(v, page) + (hp & 1) * (2 * kHalfTokens * D);
                nvalid = min(kHalfTokens, ps.L - hp * kHalfTokens);
            } else {
                const int r = hp - ps.ghp;
                base = ring_page(v, pair, r >> 1) + (r & 1) * (2 * kHalfTokens * D);
                nvalid = min(kHalfTokens, ps.Tw - r * kHalfTokens);
            }
            // keys past the valid length, and (fused step) the pair leaving the window
            const int masked_r = (FUSED && hp == drop_hp) ? drop_r : -1;
            const bool any_kill = nvalid < kHalfTokens || masked_r >= 0;
            unsigned kill = 0u;
            if (any_kill) {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (kc * 8 + e >= nvalid || kc * 8 + e == masked_r) kill |= 1u << e;
            }
            const uint16_t* kp = base + lane * 8;
            const uint16_t* vp = base + kHalfTokens * D + lane * 8;
            bf16x8 ka[2][NS], va[NB];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int sl = 0; sl < NS; ++sl)
                    ka[t][sl] = load_stream_b128(kp + (t * (D / 8) + sl * 4) * 128);
#pragma unroll
            for (int db = 0; db < NB; ++db) va[db] = load_stream_b128(vp + db * 512);
            // (Forcing all 16 loads ahead of the first MFMA with a scheduling barrier was
            // measured 2 % slower than the compiler's interleaving of loads and MFMAs.)
            attend_half_page<D>(ka, va, qb, kill, any_kill, scale_log2e, acc, m, l);
        }
    }

    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    const size_t slot = (size_t)pair * sp.slots + jj;
    // SHARED: the partial is read by another workgroup of this launch (see ticket_merge)
    if (MW == 1) {
        if (n < v.G) {
            float* pa = v.part_acc + (slot * v.G + n) * D + kc * 4;
#pragma unroll
            for (int db = 0; db < NB; ++db) {
                if (SHARED) store_device_b128(pa + db * 16, acc[db]);
                else *reinterpret_cast<f32x4*>(pa + db * 16) = acc[db];
            }
            if (kc == 0) {
                float* pm = v.part_ml + (slot * v.G + n) * 2;
                if (SHARED) {
                    store_device_b32(pm, m);
                    store_device_b32(pm + 1, l);
                } else {
                    pm[0] = m;
                    pm[1] = l;
                }
            }
        }
        return;
    }
    // the workgroup's waves meet: acc[wave][head][d] (rows kMergePad floats apart), m, l
    constexpr int kRow = D + kMergePad;
    float* s_acc = s_mem;
    float* s_m = s_mem + MW * v.G * kRow;
    float* s_l = s_m + MW * 16;
    if (n < v.G) {
        float* pa = s_acc + (wave * v.G + n) * kRow + kc * 4;
#pragma unroll
        for (int db = 0; db < NB; ++db) *reinterpret_cast<f32x4*>(pa + db * 16) = acc[db];
        if (kc == 0) {
            s_m[wave * 16 + n] = m;
            s_l[wave * 16 + n] = l;
        }
    }
    __syncthreads();
    // one partial per workgroup: with M the largest reference of the waves,
    // acc = sum_w 2^(m_w - M) acc_w,  l = sum_w 2^(m_w - M) l_w
    for (int e = threadIdx.x; e < v.G * D; e += 64 * MW) {
        const int g = e / D, d = e - g * D;
        float mw[MW], M = SPKV_NEG_INF;
#pragma unroll
        for (int w = 0; w < MW; ++w) {
            mw[w] = s_m[w * 16 + g];
            M = fmaxf(M, mw[w]);
        }
        const float m_ref = (M == SPKV_NEG_INF) ? 0.f : M;      // no key at all: every weight 0
        float a = 0.f, lsum = 0.f;
#pragma unroll
        for (int w = 0; w < MW; ++w) {
            const float sc = __builtin_amdgcn_exp2f(mw[w] - m_ref);
            a += sc * s_acc[(w * v.G + g) * kRow + d];
            lsum += sc * s_l[w * 16 + g];
        }
        float* pa = v.part_acc + (slot * v.G + g) * D + d;
        float* pm = v.part_ml + (slot * v.G + g) * 2;
        if (SHARED) {
            store_device_b32(pa, a);
            if (d == 0) {
                store_device_b32(pm, M);
                store_device_b32(pm + 1, lsum);
            }
        } else {
            *pa = a;
            if (d == 0) {
                pm[0] = M;
                pm[1] = lsum;
            }
        }
    }
}

// Inputs and outputs of the merging workgroup (modes with a ticket).
struct SpkvStepIO {
    uint16_t* out;            // [B][Hq][D]
    float* lse;               // [B][Hq] or null
    const uint16_t* k_new;    // fused step: the new token's pair and logits
    const uint16_t* v_new;
    const float* f_new;
};

// Ticket and merge.  Every workgroup of the pair calls this once, after its partial (if it
// had work) has been stored.  In the merging workgroup a thread owns eight consecutive
// floats of the pair's G x D outputs (a "unit": two float4 of one head); the waves share the
// partials round-robin, their loads go out eight partials at a time and only the cheap
// rescaling is chained; with several waves the wave results meet in LDS.
template <int D, bool STEP, int MW>
__device__ __forceinline__ void ticket_merge(const SpkvView& v, const uint16_t* __restrict__ q,
                                             float scale_log2e, SpkvSplit sp, const PairSplit& ps,
                                             int pair, float* s_mem, int* s_page, const SpkvStepIO& io) {
    constexpr int NT = 64 * MW, UPH = D / 8, U = 8, kRow = D + kMergePad;
    const int tid = threadIdx.x;
    wait_all_vmem();          // this thread's partial stores (written through) have arrived
    int ticket = 0;
    if (MW == 1) {
        if (tid == 0) ticket = atomicAdd(v.pair_ticket + pair, 1);
        ticket = __builtin_amdgcn_readfirstlane(ticket);
    } else {
        int* s_t = reinterpret_cast<int*>(s_mem);
        __syncthreads();                                     // all threads released; LDS is free
        if (tid == 0) *s_t = atomicAdd(v.pair_ticket + pair, 1);
        __syncthreads();
        ticket = *s_t;
        __syncthreads();                                     // before LDS is written again
    }
    if (ticket != sp.slots - 1) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");       // the others' partials
    if (tid == 0) v.pair_ticket[pair] = 0;                   // for the next launch

    const int b = pair / v.Hkv, h = pair - b * v.Hkv;
    const int lane = tid & 63, wave = MW == 1 ? 0 : __builtin_amdgcn_readfirstlane(tid >> 6);
    const size_t kv_row = ((size_t)b * v.Hkv + h) * D;
    const int n_part = ps.groups, NU = v.G * UPH;            // units of the pair
    const size_t slot0 = (size_t)pair * sp.slots;
    float* s_acc = s_mem;                                    // [MW][G][kRow]   (MW > 1 only)
    float* s_m = s_mem + MW * v.G * kRow;                    // [MW][16]
    float* s_l = s_m + MW * 16;

    // The finish of one unit: the new token's own term (step), normalisation, bf16, store.
    auto finish = [&](int g, int d8, bool ok, float M, float den, const f32x4 (&acc)[2]) {
        const size_t o_row = (size_t)b * v.Hq + (size_t)h * v.G + g;
        float Mt = M, w_tok = 0.f;
        f32x4 vn[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
        if (STEP) {
            // score q . k_new in fp32 (the UPH lanes of a head add up), weight sum 1, value v_new
            const uint4 qe = *reinterpret_cast<const uint4*>(q + o_row * D + d8 * 8);
            const uint4 ke = *reinterpret_cast<const uint4*>(io.k_new + kv_row + d8 * 8);
            const uint4 ve = *reinterpret_cast<const uint4*>(io.v_new + kv_row + d8 * 8);
            const unsigned qw[4] = {qe.x, qe.y, qe.z, qe.w}, kw[4] = {ke.x, ke.y, ke.z, ke.w};
            const unsigned vw[4] = {ve.x, ve.y, ve.z, ve.w};
            float dot = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                dot += __builtin_bit_cast(float, qw[e] << 16) * __builtin_bit_cast(float, kw[e] << 16);
                dot += __builtin_bit_cast(float, qw[e] & 0xffff0000u) * __builtin_bit_cast(float, kw[e] & 0xffff0000u);
                vn[e >> 1][(e & 1) * 2] = __builtin_bit_cast(float, vw[e] << 16);
                vn[e >> 1][(e & 1) * 2 + 1] = __builtin_bit_cast(float, vw[e] & 0xffff0000u);
            }
            if (!ok) dot = 0.f;
#pragma unroll
            for (int o = UPH / 2; o > 0; o >>= 1) dot += __shfl_xor(dot, o);
            const float m_tok = dot * scale_log2e;
            Mt = fmaxf(M, m_tok);
            w_tok = __builtin_amdgcn_exp2f(m_tok - Mt);
        }
        const float m_ref = (Mt == SPKV_NEG_INF) ? 0.f : Mt;
        const float sc = __builtin_amdgcn_exp2f(M - m_ref);
        const float dsum = den * sc + w_tok;
        if (ok) {
            unsigned pk[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float x0 = (acc[e >> 1][(e & 1) * 2] * sc + vn[e >> 1][(e & 1) * 2] * w_tok) / dsum;
                const float x1 = (acc[e >> 1][(e & 1) * 2 + 1] * sc + vn[e >> 1][(e & 1) * 2 + 1] * w_tok) / dsum;
                const __bf16 r0 = (__bf16)x0, r1 = (__bf16)x1;
                pk[e] = (unsigned)__builtin_bit_cast(uint16_t, r0) | ((unsigned)__builtin_bit_cast(uint16_t, r1) << 16);
            }
            *reinterpret_cast<uint4*>(io.out + o_row * D + d8 * 8) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
            if (io.lse != nullptr && d8 == 0) io.lse[o_row] = (Mt + log2f(dsum)) * 0.6931471805599453f;
        }
    };

    AppendRegs<D, NT> ar;
    if (STEP)      // the append's loads travel while the partials are merged
        ar = append_load<D, NT>(v, pair, h, b, ps.T, ps.L, io.k_new, io.v_new,
                                io.f_new[(size_t)b * v.Hkv + h], tid);

    for (int u0 = 0; u0 < NU; u0 += 64) {        // every wave: all units, its share of the partials
        const int unit = u0 + lane;
        const bool ok = unit < NU;
        const int g = ok ? unit / UPH : 0, d8 = ok ? unit - g * UPH : 0;
        float M = SPKV_NEG_INF, den = 0.f;
        f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
        for (int i0 = wave; i0 < n_part; i0 += U * MW) {
            f32x4 a[U][2];
            float2 ml[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const size_t row = (slot0 + min(i0 + u * MW, n_part - 1)) * v.G + g;   // past the end: re-read, ignored
                const float* pa = v.part_acc + row * D + d8 * 8;
                a[u][0] = *reinterpret_cast<const f32x4*>(pa);
                a[u][1] = *reinterpret_cast<const f32x4*>(pa + 4);
                ml[u] = *reinterpret_cast<const float2*>(v.part_ml + row * 2);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (i0 + u * MW < n_part) {
                    const float m_new = fmaxf(M, ml[u].x);
                    const float m_ref = (m_new == SPKV_NEG_INF) ? 0.f : m_new;   // partials with no key: weight 0
                    const float so = __builtin_amdgcn_exp2f(M - m_ref);
                    const float si = __builtin_amdgcn_exp2f(ml[u].x - m_ref);
                    den = den * so + ml[u].y * si;
                    acc[0] = acc[0] * so + a[u][0] * si;
                    acc[1] = acc[1] * so + a[u][1] * si;
                    M = m_new;
                }
            }
        }
        if (MW == 1) {
            finish(g, d8, ok, M, den, acc);
        } else if (ok) {
            float* pa = s_acc + (wave * v.G + g) * kRow + d8 * 8;
            *reinterpret_cast<f32x4*>(pa) = acc[0];
            *reinterpret_cast<f32x4*>(pa + 4) = acc[1];
            if (d8 == 0) {
                s_m[wave * 16 + g] = M;
                s_l[wave * 16 + g] = den;
            }
        }
    }
    if (MW > 1) {
        __syncthreads();
        for (int u0 = 0; u0 < NU; u0 += NT) {
            const int unit = u0 + tid;
            const bool ok = unit < NU;
            const int g = ok ? unit / UPH : 0, d8 = ok ? unit - g * UPH : 0;
            float mw[MW], M = SPKV_NEG_INF;
#pragma unroll
            for (int w = 0; w < MW; ++w) {
                mw[w] = s_m[w * 16 + g];
                M = fmaxf(M, mw[w]);
            }
            const float m_ref = (M == SPKV_NEG_INF) ? 0.f : M;
            float den = 0.f;
            f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
            for (int w = 0; w < MW; ++w) {
                const float sc = __builtin_amdgcn_exp2f(mw[w] - m_ref);
                const float* pa = s_acc + (w * v.G + g) * kRow + d8 * 8;
                acc[0] += *reinterpret_cast<const f32x4*>(pa) * sc;
                acc[1] += *reinterpret_cast<const f32x4*>(pa + 4) * sc;
                den += s_l[w * 16 + g] * sc;
            }
            finish(g, d8, ok, M, den, acc);
        }
    }
    if (STEP) append_store<D, NT>(v, pair, ps.T, ps.L, ar, tid, s_page);
}

template <int D, int MODE, int MW>
__device__ __forceinline__ void decode_split_item(const SpkvView& v, const uint16_t* __restrict__ q,
                                                  float scale_log2e, SpkvSplit sp, int wg, float* s_mem,
                                                  int* s_page, const SpkvStepIO& io) {
    constexpr bool FUSED = MODE == kSplitFusedTwo || MODE == kSplitStep;
    const int pair = wg / sp.slots;
    const int jj = wg - pair * sp.slots;
    const PairSplit ps = pair_split(v, pair, sp);
    if (MODE == kSplitFusedTwo && jj == 0 && threadIdx.x == 0) v.pair_items[pair] = ps.groups;
    constexpr bool TICKET = MODE == kSplitMerge || MODE == kSplitStep;
    if (jj < ps.groups)       // the whole workgroup
        split_compute<D, FUSED, MW, TICKET>(v, q, scale_log2e, sp, ps, pair, jj, s_mem);
    if (MODE == kSplitMerge || MODE == kSplitStep)
        ticket_merge<D, MODE == kSplitStep, MW>(v, q, scale_log2e, sp, ps, pair, s_mem, s_page, io);
}

// Merge workgroups of 16 waves instead of 4: when pairs have more than 64 partials and the
// merge launch has at most one workgroup per compute unit (few long sequences; measured on
// 4 sequences of 128k with about 150 partials per pair: 1.1 us less per step; with 39 per
// pair, 0.5 us more; with 512 merge workgroups, 3 us more).
static bool wide_merge(const SpkvView& v, const SpkvSplit& sp) {
    return sp.slots > 64 && v.n_pairs * v.G <= 256;
}

template <int D, int MODE, int MW>
__global__ __launch_bounds__(64 * MW) void spkv_decode_split(SpkvView v, const uint16_t* __restrict__ q,
                                                             float scale_log2e, SpkvSplit sp, SpkvStepIO io) {
    extern __shared__ __attribute__((aligned(16))) float s_split[];
    __shared__ int s_page;
    decode_split_item<D, MODE, MW>(v, q, scale_log2e, sp, blockIdx.x, s_split, &s_page, io);
}

// Fused step with the utility predictor (Eq. 1; the appendix builds it as Linear - SiLU -
// Linear per token): the hidden layer rides in the split launch, the output layer in the
// append workgroups of the second launch, so the gate logits of the new tokens cost no
// launch of their own.  The waves of the first ceil(pr.n_blocks / MW) workgroups of
// this launch compute partial sums of the hidden layer: wave (jb, tb, ks) takes 16 hidden
// units, 16 tokens and the ks-th of kPredictSplit ranges of d_model on MFMA 16x16x32 (W1 rows
// as A operand, tokens as the 16 columns) and stores part[ks][token][unit], without bias.
// The other workgroups are those of spkv_decode_split<D, true>.
template <int D, int MW>
__global__ __launch_bounds__(64 * MW) void spkv_decode_split_predict(SpkvView v,
                                                                const uint16_t* __restrict__ q,
                                                                float scale_log2e, SpkvSplit sp,
                                                                SpkvPredict pr) {
    extern __shared__ __attribute__((aligned(16))) float s_split[];
    const int n_pred_wg = (pr.n_blocks + MW - 1) / MW;
    if ((int)blockIdx.x >= n_pred_wg) {
        const SpkvStepIO none = {};
        decode_split_item<D, kSplitFusedTwo, MW>(v, q, scale_log2e, sp, (int)blockIdx.x - n_pred_wg,
                                                 s_split, nullptr, none);
        return;
    }
    const int unit = (int)blockIdx.x * MW + ((int)threadIdx.x >> 6);
    if (unit >= pr.n_blocks) return;
    const int n_jb = pr.d_hidden / 16;
    const int ks = unit % kPredictSplit, rest = unit / kPredictSplit;
    const int jb = rest % n_jb, tb = rest / n_jb;
    const int lane = threadIdx.x & 63, kc = lane >> 4, n = lane & 15;
    const int kq = pr.d_model / kPredictSplit;            // a multiple of 32
    const int tok = tb * 16 + n;
    const bool tok_ok = tok < v.B;
    // (columns past the last token read token 0's row; their results are never stored)
    const uint16_t* wrow = pr.w1 + (size_t)(jb * 16 + n) * pr.d_model + ks * kq + kc * 8;
    const uint16_t* xrow = pr.x + (size_t)(tok_ok ? tok : 0) * pr.d_model + ks * kq + kc * 8;
    const f32x4 acc = predictor_contract(wrow, xrow, kq);
    // lane (kc, n) holds hidden units jb * 16 + 4 kc + i of token tb * 16 + n
    if (tok_ok)
        *reinterpret_cast<f32x4*>(pr.part + ((size_t)ks * v.B + tok) * pr.d_hidden + jb * 16 + 4 * kc) = acc;
}

// One wave folds the partials of one (pair, head) into a running (max, sum, acc) triple:
// with M the running max,  acc = sum_i 2^(m_i - M) acc_i,  den = sum_i 2^(m_i - M) l_i.
// The loads of successive items are independent; only the cheap rescaling is chained.
// Lane owns E = D / 64 output elements.  The wave takes items first, first + stride, ...;
// the loads of its first eight go out before `items` is looked at (slots beyond the count
// are valid memory whose contents are then ignored), so that the round trip that fetches the
// count and the one that fetches the partials overlap.
template <int D>
__device__ __forceinline__ void fold_items(const SpkvView& v, size_t slot0, int g, int first,
                                           int stride, int slots, int items, int lane, float& mw,
                                           float& den, float (&num)[D / 64]) {
    constexpr int E = D / 64, U = 8;
    mw = SPKV_NEG_INF;
    den = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) num[e] = 0.f;
    auto fold = [&](float mi, float li, const float (&a)[E]) {
        const float m_new = fmaxf(mw, mi);
        const float m_ref = (m_new == SPKV_NEG_INF) ? 0.f : m_new;   // items with no key: weight 0
        const float so = __builtin_amdgcn_exp2f(mw - m_ref), si = __builtin_amdgcn_exp2f(mi - m_ref);
        den = den * so + li * si;
#pragma unroll
        for (int e = 0; e < E; ++e) num[e] = num[e] * so + a[e] * si;
        mw = m_new;
    };
    float m0[U], l0[U], a0[U][E];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = min(first + u * stride, slots - 1);
        const float* pm = v.part_ml + ((slot0 + i) * v.G + g) * 2;
        const float* pa = v.part_acc + ((slot0 + i) * v.G + g) * D + lane * E;
        m0[u] = pm[0];
        l0[u] = pm[1];
#pragma unroll
        for (int e = 0; e < E; ++e) a0[u][e] = pa[e];
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (first + u * stride < items) fold(m0[u], l0[u], a0[u]);
#pragma unroll 8
    for (int i = first + U * stride; i < items; i += stride) {
        const float* pm = v.part_ml + ((slot0 + i) * v.G + g) * 2;
        const float* pa = v.part_acc + ((slot0 + i) * v.G + g) * D + lane * E;
        const float mi = pm[0], li = pm[1];
        float a[E];
#pragma unroll
        for (int e = 0; e < E; ++e) a[e] = pa[e];
        fold(mi, li, a);
    }
}

// Merge the partials of one (sequence, query head):
//   out = sum_i 2^(m_i - M) acc_i / sum_i 2^(m_i - M) l_i,  lse = (M + log2(sum)) ln 2.
// One workgroup of NWM waves per (pair, head): the waves take the items round-robin, each
// lane owns D/64 output elements, and the wave results meet in LDS.  NWM = 4, or 16 (see
// wide_merge) so that every wave still gets its items in one round of loads.
template <int D, int NWM>
__global__ __launch_bounds__(64 * NWM) void spkv_decode_combine(SpkvView v, uint16_t* __restrict__ out,
                                                                float* __restrict__ lse, SpkvSplit sp) {
    constexpr int E = D / 64;
    const int pair = blockIdx.x / v.G, g = blockIdx.x - pair * v.G;
    const int b = pair / v.Hkv, h = pair - b * v.Hkv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int items = pair_split(v, pair, sp).groups;
    const size_t slot0 = (size_t)pair * sp.slots;
    __shared__ float s_m[NWM];
    __shared__ float s_den[NWM];
    __shared__ float s_acc[NWM][D];

    float mw, den, num[E];
    fold_items<D>(v, slot0, g, wave, NWM, sp.slots, items, lane, mw, den, num);
#pragma unroll
    for (int e = 0; e < E; ++e) s_acc[wave][lane * E + e] = num[e];
    if (lane == 0) {
        s_m[wave] = mw;
        s_den[wave] = den;
    }
    __syncthreads();
    if (tid < D) {
        float M = s_m[0];
#pragma unroll
        for (int wv = 1; wv < NWM; ++wv) M = fmaxf(M, s_m[wv]);
        float nsum = 0.f, dsum = 0.f;
#pragma unroll
        for (int wv = 0; wv < NWM; ++wv) {
            const float sc = __builtin_amdgcn_exp2f(s_m[wv] - M);   // 0 for a wave without items
            nsum += s_acc[wv][tid] * sc;
            dsum += s_den[wv] * sc;
        }
        const size_t o = ((size_t)b * v.Hq + (size_t)h * v.G + g);
        const __bf16 r = (__bf16)(nsum / dsum);
        out[o * D + tid] = __builtin_bit_cast(uint16_t, r);
        if (lse != nullptr && tid == 0) lse[o] = (M + log2f(dsum)) * 0.6931471805599453f;
    }
}

// Second launch of the fused step: one workgroup per (sequence, query head) merges the
// partials as spkv_decode_combine does, plus one more term for the new token itself, taken
// straight from the caller's k_new / v_new (score q . k_new in fp32, weight sum 1, value
// v_new).  n_pairs further workgroups of the same launch perform the append of the new
// token exactly as spkv_append_step does, beside the merges instead of after them.  The
// item count of a pair comes from pair_items (written by the split kernel), not from the
// counters, so no merging workgroup reads what the appends are changing.
//
// PRED (step with the utility predictor): f_new is not an input.  The append workgroup of
// (sequence b, head h) first finishes the predictor for its token and head -- hidden
// activations a_j = SiLU(b1_j + sum of the kPredictSplit partial sums the split launch left),
// logit = b2_h + sum_j W2[h, j] a_j, all in fp32 -- stores the logit for the caller and
// appends with it.
template <int D, bool PRED, int NWM>
__global__ __launch_bounds__(64 * NWM) void spkv_combine_append(SpkvView v, uint16_t* __restrict__ out,
                                                           float* __restrict__ lse, SpkvSplit sp,
                                                           const uint16_t* __restrict__ k_new,
                                                           const uint16_t* __restrict__ v_new,
                                                           const float* __restrict__ f_new,
                                                           const uint16_t* __restrict__ q,
                                                           float scale_log2e, SpkvPredict pr) {
    constexpr int E = D / 64;
    __shared__ int s_page;
    if ((int)blockIdx.x >= v.n_pairs * v.G) {                // the appends
        const int pair = blockIdx.x - v.n_pairs * v.G;
        const int b = pair / v.Hkv, h = pair - b * v.Hkv;
        const int T = v.t_pair[pair], L = v.kept_len[pair];
        float f_tok;
        if (PRED) {
            __shared__ float s_sum[NWM];
            float sum = 0.f;
            for (int j = threadIdx.x; j < pr.d_hidden; j += 64 * NWM) {
                float a = pr.b1 != nullptr ? pr.b1[j] : 0.f;
#pragma unroll
                for (int ks = 0; ks < kPredictSplit; ++ks)
                    a += pr.part[((size_t)ks * v.B + b) * pr.d_hidden + j];
                const unsigned wbits = pr.w2[(size_t)h * pr.d_hidden + j];
                sum += __builtin_bit_cast(float, wbits << 16) * (a / (1.f + __expf(-a)));   // SiLU
            }
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
            if ((threadIdx.x & 63) == 0) s_sum[threadIdx.x >> 6] = sum;
            __syncthreads();
            f_tok = pr.b2 != nullptr ? pr.b2[h] : 0.f;
#pragma unroll
            for (int wv = 0; wv < NWM; ++wv) f_tok += s_sum[wv];
            if (threadIdx.x == 0) pr.logits[(size_t)b * v.Hkv + h] = f_tok;
        } else {
            f_tok = f_new[(size_t)b * v.Hkv + h];
        }
        const AppendRegs<D> ar = append_load<D>(v, pair, h, b, T, L, k_new, v_new, f_tok, threadIdx.x);
        append_store<D>(v, pair, T, L, ar, threadIdx.x, &s_page);
        return;
    }
    const int pair = blockIdx.x / v.G, g = blockIdx.x - pair * v.G;
    const int b = pair / v.Hkv, h = pair - b * v.Hkv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int items = v.pair_items[pair];
    const size_t kv_row = ((size_t)b * v.Hkv + h) * D;
    const size_t q_row = ((size_t)b * v.Hq + (size_t)h * v.G + g) * D;
    // score of the new token for this head (every wave computes it; 6 shuffles)
    float dot = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const unsigned qe = q[q_row + lane * E + e], ke = k_new[kv_row + lane * E + e];
        dot += __builtin_bit_cast(float, qe << 16) * __builtin_bit_cast(float, ke << 16);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) dot += __shfl_xor(dot, o);
    const float m_tok = dot * scale_log2e;
    const size_t slot0 = (size_t)pair * sp.slots;
    __shared__ float s_m[NWM];
    __shared__ float s_den[NWM];
    __shared__ float s_acc[NWM][D];

    float mw, den, num[E];
    fold_items<D>(v, slot0, g, wave, NWM, sp.slots, items, lane, mw, den, num);
#pragma unroll
    for (int e = 0; e < E; ++e) s_acc[wave][lane * E + e] = num[e];
    if (lane == 0) {
        s_m[wave] = mw;
        s_den[wave] = den;
    }
    __syncthreads();
    if (tid < D) {
        float M = m_tok;
#pragma unroll
        for (int wv = 0; wv < NWM; ++wv) M = fmaxf(M, s_m[wv]);
        const float w_tok = __builtin_amdgcn_exp2f(m_tok - M);
        const unsigned ve = v_new[kv_row + tid];
        float nsum = __builtin_bit_cast(float, ve << 16) * w_tok, dsum = w_tok;
#pragma unroll
        for (int wv = 0; wv < NWM; ++wv) {
            const float sc = __builtin_amdgcn_exp2f(s_m[wv] - M);
            nsum += s_acc[wv][tid] * sc;
            dsum += s_den[wv] * sc;
        }
        const size_t o = ((size_t)b * v.Hq + (size_t)h * v.G + g);
        const __bf16 r = (__bf16)(nsum / dsum);
        out[o * D + tid] = __builtin_bit_cast(uint16_t, r);
        if (lse != nullptr && tid == 0) lse[o] = (M + log2f(dsum)) * 0.6931471805599453f;
    }
}

// ------------------------------------------------------- multi-token step (chunk)
// Up to 16 new tokens per sequence attend in one pass (speculative-decoding verification,
// prompt feed in 16-token chunks): the MFMA columns are (token i, head g) pairs, col =
// i G + g, in NQ groups of 16, so every K/V tile is still read once per (sequence, KV head).
// The cache is in the state before the chunk's append.  Long-term keys are available to
// every token of the chunk (they are at least w + 1 positions behind).  A ring key of age
// a (0 = oldest, position T - w) is inside the window of chunk token i iff a > i (the window
// indicator 0 <= t - s < w with t = T + i); otherwise it counts only if its logit passes the
// gate (Eq. 3-4).  The chunk's own keys (causal, always inside the window because the
// chunk is not longer than the window) are added by spkv_chunk_combine.
template <int D, int NQ>
__global__ __launch_bounds__(64) void spkv_chunk_split(SpkvView v, const uint16_t* __restrict__ q,
                                                       float scale_log2e, SpkvSplit sp, SpkvCu cu) {
    constexpr int NS = D / 32, NB = D / 16;
    const int pair = blockIdx.x / sp.slots;
    const int j = blockIdx.x - pair * sp.slots;
    const PairSplit ps = pair_split(v, pair, sp);
    if (j == 0 && threadIdx.x == 0) v.pair_items[pair] = ps.items;
    if (j >= ps.items) return;
    const int b = pair / v.Hkv, h = pair - b * v.Hkv;
    const int row0 = cu.v[b], n_tok = cu.v[b + 1] - row0;
    if (n_tok == 0) return;
    const int cols = n_tok * v.G;
    const int hbase = ps.nhp / ps.items, hrem = ps.nhp - hbase * ps.items;
    const int hp0 = j * hbase + min(j, hrem);
    const int hp1 = hp0 + hbase + (j < hrem ? 1 : 0);
    const int lane = threadIdx.x, kc = lane >> 4, n = lane & 15;

    bf16x8 qb[NQ][NS];
    int tok_of_col[NQ];
#pragma unroll
    for (int c = 0; c < NQ; ++c) {
        const int col = c * 16 + n;
        const int i = col / v.G, g = col - i * v.G;
        tok_of_col[c] = i;
        const uint16_t* qrow = q + ((size_t)(row0 + i) * v.Hq + (size_t)h * v.G + g) * D + kc * 8;
#pragma unroll
        for (int sl = 0; sl < NS; ++sl) {
            uint4 raw = {0u, 0u, 0u, 0u};
            if (col < cols) raw = *reinterpret_cast<const uint4*>(qrow + sl * 32);
            qb[c][sl] = __builtin_bit_cast(bf16x8, raw);
        }
    }
    f32x4 acc[NQ][NB];
    float m[NQ], l[NQ];
#pragma unroll
    for (int c = 0; c < NQ; ++c) {
        m[c] = SPKV_NEG_INF;
        l[c] = 0.f;
#pragma unroll
        for (int i = 0; i < NB; ++i) acc[c][i] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    const int32_t* pt = v.page_table + (size_t)pair * v.pt_cap;
    const float* rl = v.ring_logit + (size_t)pair * v.w;
    const int t_mod = ps.T % v.w;

    int hp = hp0;
    while (hp < hp1) {
        const int pbase = hp >> 1;
        const int my_page = pt[min(pbase + lane, v.pt_cap - 1)];
        const int hp_end = min(hp1, (pbase + 64) << 1);
        for (; hp < hp_end; ++hp) {
            const uint16_t* base;
            int nvalid;
            const bool ring = hp >= ps.ghp;
            if (!ring) {
                const int page = __builtin_amdgcn_readlane(my_page, (hp >> 1) - pbase);
                base = pool_page(v, page) + (hp & 1) * (2 * kHalfTokens * D);
                nvalid = min(kHalfTokens, ps.L - hp * kHalfTokens);
            } else {
                const int r = hp - ps.ghp;
                base = ring_page(v, pair, r >> 1) + (r & 1) * (2 * kHalfTokens * D);
                nvalid = min(kHalfTokens, ps.Tw - r * kHalfTokens);
            }
            // keys past the valid length (same for every column)
            unsigned kill_len = 0u;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (kc * 8 + e >= nvalid) kill_len |= 1u << e;
            // ring keys: age and gate of this lane's eight keys
            int age[8];
            unsigned gate_ok = 0u;
            if (ring) {
                const int x0 = (hp - ps.ghp) * kHalfTokens + kc * 8;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int x = x0 + e;
                    age[e] = ps.T >= v.w ? (x - t_mod + v.w) % v.w : x + v.w - ps.T;
                    if (kc * 8 + e < nvalid && gate_passes(v, rl[x], ps.T - v.w + age[e])) gate_ok |= 1u << e;
                }
            }
            const uint16_t* kp = base + lane * 8;
            const uint16_t* vp = base + kHalfTokens * D + lane * 8;
            bf16x8 ka[2][NS], va[NB];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int sl = 0; sl < NS; ++sl)
                    ka[t][sl] = load_stream_b128(kp + (t * (D / 8) + sl * 4) * 128);
#pragma unroll
            for (int db = 0; db < NB; ++db) va[db] = load_stream_b128(vp + db * 512);

#pragma unroll
            for (int c = 0; c < NQ; ++c) {
                unsigned kill = kill_len;
                if (ring) {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (!(age[e] > tok_of_col[c] || ((gate_ok >> e) & 1u))) kill |= 1u << e;
                }
                attend_half_page<D>(ka, va, qb[c], kill, ring || nvalid < kHalfTokens, scale_log2e,
                                    acc[c], m[c], l[c]);
            }
        }
    }

    const size_t slot = (size_t)pair * sp.slots + j;
#pragma unroll
    for (int c = 0; c < NQ; ++c) {
        float lc = l[c];
        lc += __shfl_xor(lc, 16);
        lc += __shfl_xor(lc, 32);
        const int col = c * 16 + n;
        if (col < cols) {
            float* pa = v.part_acc + ((slot * (NQ * 16) + col) * D) + kc * 4;
#pragma unroll
            for (int db = 0; db < NB; ++db) *reinterpret_cast<f32x4*>(pa + db * 16) = acc[c][db];
            if (kc == 0) {
                float* pm = v.part_ml + (slot * (NQ * 16) + col) * 2;
                pm[0] = m[c];
                pm[1] = lc;
            }
        }
    }
}

// Merge for one (pair, column = token i, head g): the split-K partials plus one term per
// chunk token j <= i taken from the caller's k / v rows (score q_i . k_j in fp32, sum 1,
// value v_j); bf16 output row cu[b] + i.  The waves share the partials and the chunk
// tokens round-robin and meet in LDS, as in spkv_decode_combine.
template <int D>
__global__ __launch_bounds__(256) void spkv_chunk_combine(SpkvView v, const uint16_t* __restrict__ q,
                                                          const uint16_t* __restrict__ k_new,
                                                          const uint16_t* __restrict__ v_new,
                                                          uint16_t* __restrict__ out,
                                                          float* __restrict__ lse, float scale_log2e,
                                                          SpkvSplit sp, SpkvCu cu, int cstride) {
    constexpr int E = D / 64;
    const int pair = blockIdx.x / cstride, col = blockIdx.x - pair * cstride;
    const int b = pair / v.Hkv, h = pair - b * v.Hkv;
    const int row0 = cu.v[b], n_tok = cu.v[b + 1] - row0;
    if (col >= n_tok * v.G) return;
    const int i = col / v.G, g = col - i * v.G;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int items = v.pair_items[pair];
    const size_t slot0 = (size_t)pair * sp.slots;
    __shared__ float s_m[4];
    __shared__ float s_den[4];
    __shared__ float s_acc[4][D];

    float mw = SPKV_NEG_INF, den = 0.f, num[E];
#pragma unroll
    for (int e = 0; e < E; ++e) num[e] = 0.f;
#pragma unroll 8
    for (int it = wave; it < items; it += 4) {
        const size_t idx = (slot0 + it) * cstride + col;
        const float mi = v.part_ml[idx * 2], li = v.part_ml[idx * 2 + 1];
        float a[E];
#pragma unroll
        for (int e = 0; e < E; ++e) a[e] = v.part_acc[idx * D + lane * E + e];
        const float m_new = fmaxf(mw, mi);
        const float m_ref = (m_new == SPKV_NEG_INF) ? 0.f : m_new;
        const float so = __builtin_amdgcn_exp2f(mw - m_ref), si = __builtin_amdgcn_exp2f(mi - m_ref);
        den = den * so + li * si;
#pragma unroll
        for (int e = 0; e < E; ++e) num[e] = num[e] * so + a[e] * si;
        mw = m_new;
    }
    // the chunk's own tokens 0..i
    const size_t q_row = ((size_t)(row0 + i) * v.Hq + (size_t)h * v.G + g) * D;
    float qf[E];
#pragma unroll
    for (int e = 0; e < E; ++e)
        qf[e] = __builtin_bit_cast(float, (unsigned)q[q_row + lane * E + e] << 16);
    for (int jt = wave; jt <= i; jt += 4) {
        const size_t kv_row = ((size_t)(row0 + jt) * v.Hkv + h) * D;
        float dot = 0.f, vj[E];
#pragma unroll
        for (int e = 0; e < E; ++e) {
            dot += qf[e] * __builtin_bit_cast(float, (unsigned)k_new[kv_row + lane * E + e] << 16);
            vj[e] = __builtin_bit_cast(float, (unsigned)v_new[kv_row + lane * E + e] << 16);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) dot += __shfl_xor(dot, o);
        const float mi = dot * scale_log2e;
        const float m_new = fmaxf(mw, mi);
        const float so = __builtin_amdgcn_exp2f(mw - m_new), si = __builtin_amdgcn_exp2f(mi - m_new);
        den = den * so + si;
#pragma unroll
        for (int e = 0; e < E; ++e) num[e] = num[e] * so + vj[e] * si;
        mw = m_new;
    }
#pragma unroll
    for (int e = 0; e < E; ++e) s_acc[wave][lane * E + e] = num[e];
    if (lane == 0) {
        s_m[wave] = mw;
        s_den[wave] = den;
    }
    __syncthreads();
    if (tid < D) {
        const float M = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));   // wave 0 has token 0
        float nsum = 0.f, dsum = 0.f;
#pragma unroll
        for (int wv = 0; wv < 4; ++wv) {
            const float sc = __builtin_amdgcn_exp2f(s_m[wv] - M);
            nsum += s_acc[wv][tid] * sc;
            dsum += s_den[wv] * sc;
        }
        const size_t o = (size_t)(row0 + i) * v.Hq + (size_t)h * v.G + g;
        const __bf16 r = (__bf16)(nsum / dsum);
        out[o * D + tid] = __builtin_bit_cast(uint16_t, r);
        if (lse != nullptr && tid == 0) lse[o] = (M + log2f(dsum)) * 0.6931471805599453f;
    }
}

template <int D, int NQ>
static hipError_t launch_chunk(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                               const uint16_t* q, uint16_t* out, float* lse, float scale_log2e,
                               SpkvSplit sp, const SpkvCu& cu, hipStream_t s) {
    const unsigned grid = (unsigned)v.n_pairs * (unsigned)sp.slots;
    spkv_chunk_split<D, NQ><<<dim3(grid), dim3(64), 0, s>>>(v, q, scale_log2e, sp, cu);
    spkv_chunk_combine<D><<<dim3(v.n_pairs * NQ * 16), dim3(256), 0, s>>>(
        v, q, k, vv, out, lse, scale_log2e, sp, cu, NQ * 16);
    return hipGetLastError();
}

hipError_t spkv_launch_decode_chunk(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                                    const uint16_t* q, uint16_t* out, float* lse, float sm_scale,
                                    SpkvSplit sp, const SpkvCu& cu, int col_groups, hipStream_t s) {
    const float sl = sm_scale * 1.4426950408889634f;
    if (v.D == 128) {
        if (col_groups <= 1) return launch_chunk<128, 1>(v, k, vv, q, out, lse, sl, sp, cu, s);
        if (col_groups == 2) return launch_chunk<128, 2>(v, k, vv, q, out, lse, sl, sp, cu, s);
        return launch_chunk<128, 4>(v, k, vv, q, out, lse, sl, sp, cu, s);
    }
    if (col_groups <= 1) return launch_chunk<64, 1>(v, k, vv, q, out, lse, sl, sp, cu, s);
    if (col_groups == 2) return launch_chunk<64, 2>(v, k, vv, q, out, lse, sl, sp, cu, s);
    return launch_chunk<64, 4>(v, k, vv, q, out, lse, sl, sp, cu, s);
}

int spkv_chunk_resident_items(int head_dim, int col_groups) {
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    hipError_t e;
    if (head_dim == 128) {
        if (col_groups <= 1) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, spkv_chunk_split<128, 1>, 64, 0);
        else if (col_groups == 2) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, spkv_chunk_split<128, 2>, 64, 0);
        else e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, spkv_chunk_split<128, 4>, 64, 0);
    } else {
        if (col_groups <= 1) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, spkv_chunk_split<64, 1>, 64, 0);
        else if (col_groups == 2) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, spkv_chunk_split<64, 2>, 64, 0);
        else e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, spkv_chunk_split<64, 4>, 64, 0);
    }
    if (e != hipSuccess || per_cu <= 0 || cus <= 0) return 0;
    return per_cu * cus;
}

// Launch of the split kernel for the call's merge width (1, 2 or 4 waves per workgroup).
template <int D, int MODE>
static void launch_split(const SpkvView& v, const uint16_t* q, float scale_log2e, SpkvSplit sp,
                         const SpkvStepIO& io, hipStream_t s) {
    const dim3 grid((unsigned)v.n_pairs * (unsigned)sp.slots);
    const size_t lds = split_lds_bytes(sp.mw, v.G, D);
    if (sp.mw == 4) spkv_decode_split<D, MODE, 4><<<grid, dim3(256), lds, s>>>(v, q, scale_log2e, sp, io);
    else if (sp.mw == 2) spkv_decode_split<D, MODE, 2><<<grid, dim3(128), lds, s>>>(v, q, scale_log2e, sp, io);
    else spkv_decode_split<D, MODE, 1><<<grid, dim3(64), 0, s>>>(v, q, scale_log2e, sp, io);
}

template <int D>
static void launch_split_predict(const SpkvView& v, const uint16_t* q, float scale_log2e,
                                 SpkvSplit sp, const SpkvPredict& pr, hipStream_t s) {
    const dim3 grid((unsigned)((pr.n_blocks + sp.mw - 1) / sp.mw) + (unsigned)v.n_pairs * (unsigned)sp.slots);
    const size_t lds = split_lds_bytes(sp.mw, v.G, D);
    if (sp.mw == 4) spkv_decode_split_predict<D, 4><<<grid, dim3(256), lds, s>>>(v, q, scale_log2e, sp, pr);
    else if (sp.mw == 2) spkv_decode_split_predict<D, 2><<<grid, dim3(128), lds, s>>>(v, q, scale_log2e, sp, pr);
    else spkv_decode_split_predict<D, 1><<<grid, dim3(64), 0, s>>>(v, q, scale_log2e, sp, pr);
}

hipError_t spkv_launch_decode(const SpkvView& v, const uint16_t* q, uint16_t* out, float* lse,
                              float sm_scale, SpkvSplit sp, bool split_only, bool one_launch,
                              hipEvent_t ev0, hipEvent_t ev1, hipStream_t s) {
    const float scale_log2e = sm_scale * 1.4426950408889634f;
    if (sp.mw != 1 && sp.mw != 2 && sp.mw != 4) return hipErrorInvalidValue;
    hipError_t e;
    if (one_launch && !split_only) {
        const SpkvStepIO io = {out, lse, nullptr, nullptr, nullptr};
        if (ev0 != nullptr && (e = hipEventRecord(ev0, s)) != hipSuccess) return e;
        if (v.D == 128) launch_split<128, kSplitMerge>(v, q, scale_log2e, sp, io, s);
        else launch_split<64, kSplitMerge>(v, q, scale_log2e, sp, io, s);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        if (ev1 != nullptr && (e = hipEventRecord(ev1, s)) != hipSuccess) return e;
        return hipSuccess;
    }
    const SpkvStepIO none = {};
    if (ev0 != nullptr && (e = hipEventRecord(ev0, s)) != hipSuccess) return e;
    if (v.D == 128) launch_split<128, kSplitPlain>(v, q, scale_log2e, sp, none, s);
    else launch_split<64, kSplitPlain>(v, q, scale_log2e, sp, none, s);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (ev1 != nullptr && (e = hipEventRecord(ev1, s)) != hipSuccess) return e;
    if (split_only) return hipSuccess;
    const dim3 grid2(v.n_pairs * v.G);
    if (wide_merge(v, sp)) {
        if (v.D == 128) spkv_decode_combine<128, 16><<<grid2, dim3(1024), 0, s>>>(v, out, lse, sp);
        else spkv_decode_combine<64, 16><<<grid2, dim3(1024), 0, s>>>(v, out, lse, sp);
    } else {
        if (v.D == 128) spkv_decode_combine<128, 4><<<grid2, dim3(256), 0, s>>>(v, out, lse, sp);
        else spkv_decode_combine<64, 4><<<grid2, dim3(256), 0, s>>>(v, out, lse, sp);
    }
    return hipGetLastError();
}

// One-wave work items the device holds at once (the registers decide, so the count is the
// same for every merge width).
int spkv_split_resident_items(int head_dim) {
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    const hipError_t e =
        head_dim == 128
            ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, spkv_decode_split<128, kSplitStep, 1>, 64, 0)
            : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, spkv_decode_split<64, kSplitStep, 1>, 64, 0);
    if (e != hipSuccess || per_cu <= 0 || cus <= 0) return 0;
    return per_cu * cus;
}

hipError_t spkv_launch_decode_step(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                                   const float* f, const uint16_t* q, uint16_t* out, float* lse,
                                   float sm_scale, SpkvSplit sp, bool one_launch, hipStream_t s) {
    const float scale_log2e = sm_scale * 1.4426950408889634f;
    if (sp.mw != 1 && sp.mw != 2 && sp.mw != 4) return hipErrorInvalidValue;
    if (one_launch) {
        const SpkvStepIO io = {out, lse, k, vv, f};
        if (v.D == 128) launch_split<128, kSplitStep>(v, q, scale_log2e, sp, io, s);
        else launch_split<64, kSplitStep>(v, q, scale_log2e, sp, io, s);
        return hipGetLastError();
    }
    const SpkvStepIO no_io = {};
    const SpkvPredict none = {};
    const dim3 grid2(v.n_pairs * v.G + v.n_pairs);
    const bool wide = wide_merge(v, sp);
    if (v.D == 128) {
        launch_split<128, kSplitFusedTwo>(v, q, scale_log2e, sp, no_io, s);
        if (wide) spkv_combine_append<128, false, 16><<<grid2, dim3(1024), 0, s>>>(v, out, lse, sp, k, vv, f, q, scale_log2e, none);
        else spkv_combine_append<128, false, 4><<<grid2, dim3(256), 0, s>>>(v, out, lse, sp, k, vv, f, q, scale_log2e, none);
    } else {
        launch_split<64, kSplitFusedTwo>(v, q, scale_log2e, sp, no_io, s);
        if (wide) spkv_combine_append<64, false, 16><<<grid2, dim3(1024), 0, s>>>(v, out, lse, sp, k, vv, f, q, scale_log2e, none);
        else spkv_combine_append<64, false, 4><<<grid2, dim3(256), 0, s>>>(v, out, lse, sp, k, vv, f, q, scale_log2e, none);
    }
    return hipGetLastError();
}

int spkv_predict_blocks(int n_tokens, int d_hidden) {
    return (d_hidden / 16) * ((n_tokens + 15) / 16) * kPredictSplit;
}

hipError_t spkv_launch_decode_step_predict(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                                           const uint16_t* q, uint16_t* out, float* lse,
                                           float sm_scale, SpkvSplit sp, SpkvPredict pr,
                                           hipStream_t s) {
    const float scale_log2e = sm_scale * 1.4426950408889634f;
    if (sp.mw != 1 && sp.mw != 2 && sp.mw != 4) return hipErrorInvalidValue;
    pr.n_blocks = spkv_predict_blocks(v.B, pr.d_hidden);
    const dim3 grid2(v.n_pairs * v.G + v.n_pairs);
    const bool wide = wide_merge(v, sp);
    if (v.D == 128) {
        launch_split_predict<128>(v, q, scale_log2e, sp, pr, s);
        if (wide) spkv_combine_append<128, true, 16><<<grid2, dim3(1024), 0, s>>>(v, out, lse, sp, k, vv, nullptr, q, scale_log2e, pr);
        else spkv_combine_append<128, true, 4><<<grid2, dim3(256), 0, s>>>(v, out, lse, sp, k, vv, nullptr, q, scale_log2e, pr);
    } else {
        launch_split_predict<64>(v, q, scale_log2e, sp, pr, s);
        if (wide) spkv_combine_append<64, true, 16><<<grid2, dim3(1024), 0, s>>>(v, out, lse, sp, k, vv, nullptr, q, scale_log2e, pr);
        else spkv_combine_append<64, true, 4><<<grid2, dim3(256), 0, s>>>(v, out, lse, sp, k, vv, nullptr, q, scale_log2e, pr);
    }
    return hipGetLastError();
}
