// Write path of the SP-KV cache on gfx950: zero fill and copies, the append of one token per
// sequence (fused gate + evict + ring write), the bulk append (ballot + mbcnt stream
// compaction in stable order), sequence release and the read-back of kept positions.
//
// Gate: Eq. 2 of the paper taken on the logit, z = 1[f >= theta].  The window ring holds
// exactly the keys with 0 <= t - s < w and the long-term pages exactly the gated-on keys with
// t - s >= w (Eq. 3-4), so the two sets are disjoint and their union is what Eq. 5 attends to.
#include "spkv_device.h"

// ------------------------------------------------------------------------ zero fill
__global__ __launch_bounds__(256) void spkv_fill_zero(uint4* p, size_t n16) {
    const uint4 z = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = z;
}

hipError_t spkv_launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    spkv_fill_zero<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(static_cast<uint4*>(p), n16);
    return hipGetLastError();
}

// ------------------------------------------------------------- plain copy (reference)
__global__ __launch_bounds__(256) void spkv_plain_copy(uint4* __restrict__ d,
                                                       const uint4* __restrict__ s, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16;
         i += (size_t)gridDim.x * blockDim.x)
        d[i] = s[i];
}

hipError_t spkv_launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
    const size_t n16 = bytes / 16;
    if (n16 == 0) return hipSuccess;
    size_t blocks = (n16 + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    spkv_plain_copy<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(
        static_cast<uint4*>(dst), static_cast<const uint4*>(src), n16);
    return hipGetLastError();
}

// ------------------------------------------------- plain streaming read (reference)
// The memory side of the decode kernel and nothing else: one-wave workgroups, each reading
// its share of the launch's 16 KB chunks with sixteen non-temporal 1 KB wave-wide loads per
// chunk (the half-page access pattern) and storing 1 KB at the end (as a work item stores its
// partial result).  Chunk c of the launch lies in run c / chunks_per_run; run i of the launch
// is run ((first_run + i) * stride) mod total_runs of the region, so with a stride coprime to
// total_runs successive launches read distinct, scattered runs.
__global__ __launch_bounds__(64) void spkv_plain_read(const uint16_t* __restrict__ src,
                                                      long long total_runs, int chunks_per_run,
                                                      long long first_run, long long n_chunks,
                                                      long long stride, uint4* __restrict__ sink) {
    const long long g = blockIdx.x, n = gridDim.x;
    const long long c0 = g * n_chunks / n, c1 = (g + 1) * n_chunks / n;
    const int lane = threadIdx.x;
    typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (long long c = c0; c < c1; ++c) {
        const long long i = c / chunks_per_run;
        const int within = (int)(c - i * chunks_per_run);
        const long long run = (long long)(((unsigned long long)(first_run + i) * (unsigned long long)stride) %
                                          (unsigned long long)total_runs);
        const uint16_t* base = src + ((size_t)run * chunks_per_run + within) * 8192 + lane * 8;
        u32x4 x[16];
#pragma unroll
        for (int t = 0; t < 16; ++t)
            x[t] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + t * 512));
#pragma unroll
        for (int t = 0; t < 16; ++t) acc ^= x[t];
    }
    sink[(size_t)g * 64 + lane] = make_uint4(acc.x, acc.y, acc.z, acc.w);
}

hipError_t spkv_launch_read(const void* src, long long total_runs, int chunks_per_run,
                            long long first_run, long long n_runs, long long stride,
                            int n_workgroups, void* sink, hipStream_t s) {
    spkv_plain_read<<<dim3((unsigned)n_workgroups), dim3(64), 0, s>>>(
        static_cast<const uint16_t*>(src), total_runs, chunks_per_run, first_run,
        n_runs * chunks_per_run, stride, static_cast<uint4*>(sink));
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void spkv_copy_rows(int32_t* __restrict__ dst,
                                                      const int32_t* __restrict__ src, int rows,
                                                      int src_width, int dst_width) {
    const size_t n = (size_t)rows * src_width;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const size_t r = i / src_width, c = i - r * src_width;
        dst[r * dst_width + c] = src[i];
    }
}

hipError_t spkv_launch_copy_rows(int32_t* dst, const int32_t* src, int rows, int src_width,
                                 int dst_width, hipStream_t s) {
    const size_t n = (size_t)rows * src_width;
    if (n == 0) return hipSuccess;
    const size_t blocks = std::min<size_t>((n + 255) / 256, 256 * 16);
    spkv_copy_rows<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(dst, src, rows, src_width, dst_width);
    return hipGetLastError();
}

template <int D>
__global__ __launch_bounds__(D) void spkv_append_step(SpkvView v, const uint16_t* __restrict__ k,
                                                      const uint16_t* __restrict__ vv,
                                                      const float* __restrict__ f, SpkvCu cu) {
    const int pair = blockIdx.x;
    const int b = pair / v.Hkv, h = pair - b * v.Hkv;
    const int row = cu.v[b];
    if (cu.v[b + 1] - row == 0) return;
    __shared__ int s_page;
    const int T = v.t_pair[pair];
    const int L = v.kept_len[pair];
    const AppendRegs<D> r =
        append_load<D>(v, pair, h, row, T, L, k, vv, f[(size_t)row * v.Hkv + h], threadIdx.x);
    append_store<D>(v, pair, T, L, r, threadIdx.x, &s_page);
}

hipError_t spkv_launch_append_step(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                                   const float* f, const SpkvCu& cu, hipStream_t s) {
    if (v.D == 128)
        spkv_append_step<128><<<dim3(v.n_pairs), dim3(128), 0, s>>>(v, k, vv, f, cu);
    else
        spkv_append_step<64><<<dim3(v.n_pairs), dim3(64), 0, s>>>(v, k, vv, f, cu);
    return hipGetLastError();
}

// ----------------------------------------------------- write path, many tokens (bulk)
// For (sequence, head) with n new tokens, T_old stored: positions that leave the window
// are [max(0, T_old - w), T_old + n - w).  Those below T_old sit in the ring (<= w of
// them, handled by spkv_bulk_ring); the others are new tokens j in [0, n - w) that enter
// and leave the window within this call (handled per 256-token segment, one token per
// thread).  The last min(n, w) new tokens land in the ring.  Long-term order is ascending
// position: ring-evicted first, then new tokens; ranks come from ballot + mbcnt prefix
// sums inside a wave, popcounts across the four waves of a segment, and a scan of the
// per-segment counts across segments.
//
// Rows are moved 16 at a time per workgroup: 16 lanes per row, each lane one 16-byte K
// chunk and the 8 V elements of the same head-dim range (loads coalesced per row; the V
// elements go out as 2-byte stores at 16-byte stride, which is what the page layout asks).

// Per-pair scratch written by spkv_bulk_ring for spkv_bulk_scatter.
struct BulkInfo {
    int32_t T_old;        // tokens held before this call
    int32_t new_base;     // long-term index of the first kept NEW token (after ring-evicted ones)
    int32_t ok;           // 0: capacity error, the call writes nothing more for this pair
    int32_t pad[5];
};

// Lane (r = lane / 16, c = lane % 16) moves chunk c of one row into row dk of page dp.
template <int D>
__device__ __forceinline__ void store_row_chunk(uint16_t* dp, int dk, int c, uint4 kk, uint4 vv) {
    *reinterpret_cast<uint4*>(dp + spkv_k_off(D, dk, c * 8)) = kk;
    uint16_t* vd = dp + spkv_v_off(D, dk, c * 8);      // element e of the chunk is 8 e further
    const unsigned w[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
    for (int e = 0; e < 8; ++e) vd[e * 8] = (uint16_t)(w[e >> 1] >> ((e & 1) * 16));
}

// Stage 1: per (segment, pair): how many of the segment's new tokens pass the gate, and how
// many of those also leave the window within this call (j < n - w).
__global__ __launch_bounds__(256) void spkv_bulk_count(SpkvView v, const float* __restrict__ f,
                                                       SpkvCu cu) {
    const int pair = blockIdx.y, seg = blockIdx.x;
    const int b = pair / v.Hkv, h = pair - b * v.Hkv;
    const int n = cu.v[b + 1] - cu.v[b];
    const int n_ev = max(0, n - v.w);
    const int j = seg * kSegTokens + (int)threadIdx.x;
    if (seg * kSegTokens >= n) return;
    __shared__ int s_ev[4], s_on[4];
    const bool on = j < n && gate_passes(v, f[((size_t)cu.v[b] + j) * v.Hkv + h], v.t_pair[pair] + j);
    const int c_on = __popcll(__ballot(on));
    const int c_ev = __popcll(__ballot(on && j < n_ev));
    if (lane_id() == 0) {
        s_on[threadIdx.x >> 6] = c_on;
        s_ev[threadIdx.x >> 6] = c_ev;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        v.seg_count[(size_t)pair * v.n_seg_cap + seg] = s_ev[0] + s_ev[1] + s_ev[2] + s_ev[3];
        v.seg_on[(size_t)pair * v.n_seg_cap + seg] = s_on[0] + s_on[1] + s_on[2] + s_on[3];
    }
}

// Block-wide exclusive scan of one int per thread (256 threads); returns the exclusive
// prefix and the block total.  s_w: 4 ints of shared memory.
__device__ __forceinline__ int block_excl_scan(int x, int* s_w, int& total) {
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    int incl = x;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(incl, o);
        if (lane >= o) incl += t;
    }
    __syncthreads();
    if (lane == 63) s_w[wave] = incl;
    __syncthreads();
    int woff = 0;
    total = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (i < wave) woff += s_w[i];
        total += s_w[i];
    }
    return woff + incl - x;
}

// Stage 2: one workgroup per pair.  Counts the pairs leaving the ring that are kept,
// turns the segment counts into offsets, allocates every page the call needs with one
// allocation per page, publishes the new lengths, then moves the kept ring rows.
//
// prefix (may be null; used by the prefill attention): for the new token i of the call, at
// position t = T_old + i, prefix[(row of token i) * H_kv + h] = number of long-term entries,
// after this call, whose position is <= t - w -- the entries available to query t outside
// its window (the list is in ascending position, so they are a prefix of it).  Stage 2
// writes the tokens whose t - w is a ring position, stage 3 the others; tokens with
// t - w < 0 get no entry (their count is 0).
//
// SMALL: every sequence brings at most min(w, 256) tokens, so no new token leaves the window
// within the call and this launch is the whole append: it also counts the gate-on tokens from
// the logits (stage 1's job otherwise) and, once the kept rows have left the ring, writes
// the new tokens into it (stage 3's job otherwise).
//
// COUNT: chunks of at most kCountSegs segments per sequence -- this launch also does stage 1's
// job for its pair (the per-segment counts from the logits, every wave's popcounts parked in
// LDS and summed after one barrier), so that the call is two launches instead of three.
constexpr int kCountSegs = 16;
template <int D, bool SMALL, bool COUNT>
__global__ __launch_bounds__(256) void spkv_bulk_ring(SpkvView v, SpkvCu cu, int32_t* prefix,
                                                      const uint16_t* __restrict__ k,
                                                      const uint16_t* __restrict__ vv,
                                                      const float* __restrict__ f) {
    const int pair = blockIdx.x;
    const int b = pair / v.Hkv;
    const int n = cu.v[b + 1] - cu.v[b];
    if (n == 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int T_old = v.t_pair[pair], T_new = T_old + n, L_old = v.kept_len[pair];
    const int r0 = max(0, T_old - v.w);
    const int r1 = min(T_old, max(0, T_new - v.w));
    const int nr = max(0, r1 - r0);
    const int n_ev = max(0, n - v.w);
    const int nseg = (n_ev + kSegTokens - 1) / kSegTokens;
    const float* rl = v.ring_logit + (size_t)pair * v.w;
    int32_t* sc = v.seg_count + (size_t)pair * v.n_seg_cap;
    __shared__ int s_w[4];
    __shared__ BulkInfo s_bi;
    __shared__ uint16_t s_list[256];
    __shared__ int s_seg[COUNT ? kCountSegs : 1][4][2];

    // the ring logits of the first 256 leaving positions travel with the segments' logits
    const float rl_first = tid < nr ? rl[(r0 + tid) % v.w] : 0.f;
    if (COUNT) {          // stage 1 for this pair: per segment and wave, kept-and-leaving / gate-on
        const int hh = pair - b * v.Hkv, nseg_all = (n + kSegTokens - 1) / kSegTokens;
        float fv[kCountSegs];           // every segment's logit of this thread, loads issued together
#pragma unroll
        for (int sg = 0; sg < kCountSegs; ++sg) {
            const int j = sg * kSegTokens + tid;
            fv[sg] = (sg < nseg_all && j < n) ? f[((size_t)cu.v[b] + j) * v.Hkv + hh] : 0.f;
        }
#pragma unroll
        for (int sg = 0; sg < kCountSegs; ++sg) {
            if (sg < nseg_all) {
                const int j = sg * kSegTokens + tid;
                const bool on = j < n && gate_passes(v, fv[sg], T_old + j);
                const int c_on = __popcll(__ballot(on));
                const int c_ev = __popcll(__ballot(on && j < n_ev));
                if (lane == 0) {
                    s_seg[sg][wave][0] = c_ev;
                    s_seg[sg][wave][1] = c_on;
                }
            }
        }
        __syncthreads();
        if (tid < nseg_all) {
            sc[tid] = s_seg[tid][0][0] + s_seg[tid][1][0] + s_seg[tid][2][0] + s_seg[tid][3][0];
            v.seg_on[(size_t)pair * v.n_seg_cap + tid] =
                s_seg[tid][0][1] + s_seg[tid][1][1] + s_seg[tid][2][1] + s_seg[tid][3][1];
        }
        __threadfence_block();
        __syncthreads();
    }

    // (a) how many ring pairs are kept
    int cnt = 0;
    for (int base = 0; base < nr; base += 256) {
        const int idx = base + tid;
        const bool flag = idx < nr && gate_passes(v, base == 0 ? rl_first : rl[(r0 + idx) % v.w], r0 + idx);
        cnt += __popcll(__ballot(flag));
    }
    if (lane == 0) s_w[wave] = cnt;
    __syncthreads();
    const int ring_kept = s_w[0] + s_w[1] + s_w[2] + s_w[3];

    // (b) segment counts -> exclusive offsets (in place)
    int carry = 0;
    for (int base = 0; base < nseg; base += 256) {
        const int i = base + tid;
        const int c = i < nseg ? sc[i] : 0;
        int tot;
        const int ex = block_excl_scan(c, s_w, tot);
        if (i < nseg) sc[i] = carry + ex;
        carry += tot;
    }
    const int total_new = ring_kept + carry;

    // gate-on count of the call (Eq. 8 numerator), summed here so that no kernel needs
    // same-address atomics
    {
        int on = 0;
        if (SMALL) {
            const bool flag = tid < n && gate_passes(v, f[((size_t)cu.v[b] + tid) * v.Hkv + (pair - b * v.Hkv)],
                                                     T_old + tid);
            on = flag ? 1 : 0;
        } else {
            const int nseg_all = (n + kSegTokens - 1) / kSegTokens;
            const int32_t* so = v.seg_on + (size_t)pair * v.n_seg_cap;
            for (int i = tid; i < nseg_all; i += 256) on += so[i];
        }
        for (int o = 32; o > 0; o >>= 1) on += __shfl_xor(on, o);
        __syncthreads();
        if (lane == 0) s_w[wave] = on;
        __syncthreads();
        if (tid == 0) v.gate_on[pair] += s_w[0] + s_w[1] + s_w[2] + s_w[3];
    }

    // (c) pages: all the call's pages of this pair in one allocation; the table entries are
    //     visible to the whole workgroup after the barrier and to stage 3 after the launch
    const int first = (L_old + kPageTokens - 1) / kPageTokens;
    const int last = (L_old + total_new + kPageTokens - 1) / kPageTokens;
    const int need = last <= v.pt_cap ? last - first : 0;
    int bad = last > v.pt_cap ? 1 : 0;
    __shared__ PageBatch s_pb;
    if (tid == 0) s_pb = alloc_page_batch(v, need);
    __syncthreads();
    for (int i = tid; i < need; i += 256) {
        const int page = batch_page(v, s_pb, i);
        if (page < 0) bad = 1;
        else v.page_table[(size_t)pair * v.pt_cap + first + i] = page;
    }
    const int any_bad = __syncthreads_or(bad);
    if (tid == 0) {
        if (any_bad) *v.err_flag = 1;
        s_bi.T_old = T_old;
        s_bi.new_base = L_old + ring_kept;
        s_bi.ok = any_bad ? 0 : 1;
        *reinterpret_cast<BulkInfo*>(v.bulk_info + (size_t)pair * 8) = s_bi;
        if (!any_bad) v.kept_len[pair] = L_old + total_new;
        v.t_pair[pair] = T_new;
    }
    __threadfence_block();
    __syncthreads();
    if (any_bad) return;
    const int32_t* pt = v.page_table + (size_t)pair * v.pt_cap;

    // (d) move the kept ring rows, 256 ring positions at a time
    int done = 0;
    for (int base = 0; base < nr; base += 256) {
        const int idx = base + tid;
        const bool flag = idx < nr && gate_passes(v, base == 0 ? rl_first : rl[(r0 + idx) % v.w], r0 + idx);
        int tot;
        const int rank = block_excl_scan(flag ? 1 : 0, s_w, tot);
        if (flag) s_list[rank] = (uint16_t)tid;
        if (prefix != nullptr && idx < nr) {
            const int i = r0 + idx + v.w - T_old;      // the new token whose t - w is this position
            prefix[((size_t)cu.v[b] + i) * v.Hkv + (pair - b * v.Hkv)] = L_old + done + rank + (flag ? 1 : 0);
        }
        __syncthreads();
        const int c = lane & 15;
        // four rows per lane at a time: all their loads go out before the first store
        for (int rb = wave * 4; rb < tot; rb += 64) {
            uint4 kk[4], vl[4];
            int sv[4], page[4];
            float lg[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int r = rb + u * 16 + (lane >> 4);
                sv[u] = -1;
                if (r < tot && c < D / 8) {
                    const int s = r0 + base + s_list[r];
                    const int slot = s % v.w;
                    const uint16_t* sp = ring_page(v, pair, slot >> 6);
                    const int sk = slot & 63;
                    kk[u] = *reinterpret_cast<const uint4*>(sp + spkv_k_off(D, sk, c * 8));
                    const uint16_t* vs = sp + spkv_v_off(D, sk, c * 8);
                    unsigned w[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        w[e] = (unsigned)vs[(2 * e) * 8] | ((unsigned)vs[(2 * e + 1) * 8] << 16);
                    vl[u] = make_uint4(w[0], w[1], w[2], w[3]);
                    page[u] = pt[(L_old + done + r) >> 6];
                    lg[u] = rl[slot];
                    sv[u] = s;
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (sv[u] >= 0) {
                    const int gi = L_old + done + rb + u * 16 + (lane >> 4);
                    store_row_chunk<D>(pool_page(v, page[u]), gi & 63, c, kk[u], vl[u]);
                    if (c == 0) {
                        v.pos_pool[(size_t)page[u] * kPageTokens + (gi & 63)] = sv[u];
                        v.logit_pool[(size_t)page[u] * kPageTokens + (gi & 63)] = lg[u];
                    }
                }
            }
        }
        done += tot;
        __syncthreads();
    }
    if (SMALL) {        // the new tokens into the ring slots the oldest pairs have just left
        const int h = pair - b * v.Hkv, row0 = cu.v[b], c = lane & 15;
        for (int rb = wave * 4; rb < n; rb += 16) {
            const int jj = rb + (lane >> 4);
            if (jj < n && c < D / 8) {
                const int slot = (T_old + jj) % v.w;
                const size_t src = ((size_t)(row0 + jj) * v.Hkv + h) * D + c * 8;
                const uint4 kk = *reinterpret_cast<const uint4*>(k + src);
                const uint4 vl = *reinterpret_cast<const uint4*>(vv + src);
                store_row_chunk<D>(ring_page(v, pair, slot >> 6), slot & 63, c, kk, vl);
                if (c == 0)
                    v.ring_logit[(size_t)pair * v.w + slot] = f[((size_t)row0 + jj) * v.Hkv + h];
            }
        }
    }
}

// Stage 3: per (256-token segment, pair).  Thread i owns token j0 + i: gate flag, rank
// (mbcnt inside the wave + the popcounts of the lower waves + the segment offset from
// stage 2); the kept tokens' indices are compacted into LDS and their rows moved in groups
// of eight consecutive destination rows (whole 16-byte V units, transposed through LDS),
// stragglers row by row; the last min(n, w) tokens of the call are written into the ring.
// The last min(n, w) tokens of the call go into the ring: workgroup rb of the ring part takes
// the ring slots [32 rb, 32 rb + 32), a wave eight consecutive slots -- one 16-byte V unit per
// head-dim element.  Slot s receives the newest position p < T_new with p mod w = s if the call
// brought it (p >= T_new - min(n, w)).  A unit whose eight slots are all written goes out as
// whole 16-byte units, transposed through LDS; otherwise the written rows go one by one.
template <int D>
__device__ __forceinline__ void bulk_ring_rows(const SpkvView& v, const uint16_t* __restrict__ k,
                                               const uint16_t* __restrict__ vv,
                                               const float* __restrict__ f, int pair, int h, int row0,
                                               int n, int T_old, int rb, uint16_t (*s_rows)[D],
                                               int lane, int wave) {
    const int s0 = rb * kHalfTokens + wave * 8;
    if (s0 >= v.w) return;
    const int T_new = T_old + n, m = min(n, v.w), c = lane & 15;
    // token index (row of the call) landing in slot s, or -1
    auto token_of = [&](int s) -> int {
        if (s >= v.w) return -1;
        const int p = T_new - 1 - ((T_new - 1 - s) % v.w + v.w) % v.w;
        return p >= T_new - m ? p - T_old : -1;
    };
    bool all = true;
#pragma unroll
    for (int r = 0; r < 8; ++r) all = all && token_of(s0 + r) >= 0;
    uint16_t* dp = ring_page(v, pair, s0 >> 6);
    const int dk0 = s0 & 63;
    uint4 kk[2], vl[2];
    int jj[2];
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        jj[pass] = token_of(s0 + pass * 4 + (lane >> 4));
        kk[pass] = make_uint4(0u, 0u, 0u, 0u);
        vl[pass] = make_uint4(0u, 0u, 0u, 0u);
        if (jj[pass] >= 0 && c < D / 8) {
            const size_t src = ((size_t)(row0 + jj[pass]) * v.Hkv + h) * D + c * 8;
            kk[pass] = *reinterpret_cast<const uint4*>(k + src);
            vl[pass] = *reinterpret_cast<const uint4*>(vv + src);
        }
    }
    if (lane < 8) {
        const int j = token_of(s0 + lane);
        if (j >= 0) v.ring_logit[(size_t)pair * v.w + s0 + lane] = f[((size_t)row0 + j) * v.Hkv + h];
    }
    if (all) {
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int row = pass * 4 + (lane >> 4);
            if (c < D / 8) {
                *reinterpret_cast<uint4*>(dp + spkv_k_off(D, dk0 + row, c * 8)) = kk[pass];
                *reinterpret_cast<uint4*>(&s_rows[row][c * 8]) = vl[pass];
            }
        }
        __builtin_amdgcn_wave_barrier();
        store_v_units<D>(dp, dk0, s_rows, lane);
    } else {
#pragma unroll
        for (int pass = 0; pass < 2; ++pass)
            if (jj[pass] >= 0 && c < D / 8)
                store_row_chunk<D>(dp, dk0 + pass * 4 + (lane >> 4), c, kk[pass], vl[pass]);
    }
}

template <int D>
__global__ __launch_bounds__(256) void spkv_bulk_scatter(SpkvView v, const uint16_t* __restrict__ k,
                                                         const uint16_t* __restrict__ vv,
                                                         const float* __restrict__ f, SpkvCu cu,
                                                         int32_t* prefix, int segs_all) {
    const int pair = blockIdx.y, seg = blockIdx.x;
    const int b = pair / v.Hkv, h = pair - b * v.Hkv;
    const int row0 = cu.v[b];
    const int n = cu.v[b + 1] - row0;
    const int j0 = seg * kSegTokens;
    if (n == 0 || (seg < segs_all && j0 >= n)) return;
    const BulkInfo bi = *reinterpret_cast<const BulkInfo*>(v.bulk_info + (size_t)pair * 8);
    if (bi.ok == 0) return;
    const int n_ev = max(0, n - v.w);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, c = lane & 15;
    __shared__ int s_cnt[4];
    __shared__ uint16_t s_list[256];
    __shared__ __attribute__((aligned(16))) uint16_t s_v[4][8][D];
    if (seg >= segs_all) {      // the ring part of the grid: independent of the segments
        bulk_ring_rows<D>(v, k, vv, f, pair, h, row0, n, bi.T_old, seg - segs_all, s_v[wave], lane, wave);
        return;
    }

    const int j = j0 + tid;
    const bool on = j < n && gate_passes(v, f[((size_t)row0 + j) * v.Hkv + h], bi.T_old + j);
    const bool ev = on && j < n_ev;
    const unsigned long long mask = __ballot(ev);
    if (lane == 0) s_cnt[wave] = __popcll(mask);
    __syncthreads();
    int woff = 0, total = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (i < wave) woff += s_cnt[i];
        total += s_cnt[i];
    }
    if (ev) s_list[woff + mbcnt64(mask)] = (uint16_t)tid;
    if (prefix != nullptr && j < n_ev)       // token j leaves the window of token j + w
        prefix[((size_t)row0 + j + v.w) * v.Hkv + h] =
            bi.new_base + v.seg_count[(size_t)pair * v.n_seg_cap + seg] + woff + mbcnt64(mask) + (ev ? 1 : 0);
    __syncthreads();

    if (total > 0) {
        const int g0 = bi.new_base + v.seg_count[(size_t)pair * v.n_seg_cap + seg];
        const int32_t* pt = v.page_table + (size_t)pair * v.pt_cap;
        const int gend = g0 + total;
        const int ga = min(gend, (g0 + 7) & ~7);   // destination indices [ga, gb) are whole
        const int gb = max(ga, gend & ~7);         // groups of 8 aligned to 8: whole V units

        // Whole groups, one wave each: K chunks go straight out; the eight V rows meet in
        // LDS and leave as 16-byte units (eight keys of one head-dim element).
        for (int G8 = ga + wave * 8; G8 < gb; G8 += 32) {
            const int page = pt[G8 >> 6];
            uint16_t* dp = pool_page(v, page);
            const int dk0 = G8 & 63;
#pragma unroll
            for (int pass = 0; pass < 2; ++pass) {
                const int row = pass * 4 + (lane >> 4);
                if (c < D / 8) {
                    const int jj = j0 + s_list[G8 - g0 + row];
                    const size_t src = ((size_t)(row0 + jj) * v.Hkv + h) * D + c * 8;
                    const uint4 kk = *reinterpret_cast<const uint4*>(k + src);
                    const uint4 vl = *reinterpret_cast<const uint4*>(vv + src);
                    *reinterpret_cast<uint4*>(dp + spkv_k_off(D, dk0 + row, c * 8)) = kk;
                    *reinterpret_cast<uint4*>(&s_v[wave][row][c * 8]) = vl;
                }
            }
            __builtin_amdgcn_wave_barrier();
            if (lane < D / 2) {
                unsigned dw[8];
#pragma unroll
                for (int r = 0; r < 8; ++r)
                    dw[r] = *reinterpret_cast<const unsigned*>(&s_v[wave][r][2 * lane]);
                uint4 lo, hi;
                lo.x = (dw[0] & 0xffffu) | (dw[1] << 16);
                lo.y = (dw[2] & 0xffffu) | (dw[3] << 16);
                lo.z = (dw[4] & 0xffffu) | (dw[5] << 16);
                lo.w = (dw[6] & 0xffffu) | (dw[7] << 16);
                hi.x = (dw[0] >> 16) | (dw[1] & 0xffff0000u);
                hi.y = (dw[2] >> 16) | (dw[3] & 0xffff0000u);
                hi.z = (dw[4] >> 16) | (dw[5] & 0xffff0000u);
                hi.w = (dw[6] >> 16) | (dw[7] & 0xffff0000u);
                uint16_t* vd = dp + spkv_v_off(D, dk0, 2 * lane);   // unit of d = 2 lane; d + 1 follows
                *reinterpret_cast<uint4*>(vd) = lo;
                *reinterpret_cast<uint4*>(vd + 8) = hi;
            }
            if (lane < 8) {
                const int jj = j0 + s_list[G8 - g0 + lane];
                v.pos_pool[(size_t)page * kPageTokens + dk0 + lane] = bi.T_old + jj;
                v.logit_pool[(size_t)page * kPageTokens + dk0 + lane] = f[((size_t)row0 + jj) * v.Hkv + h];
            }
            __builtin_amdgcn_wave_barrier();
        }
        // The rows before the first and after the last whole group, one row per 16 lanes,
        // V elements as 2-byte stores.
        const int n_head = ga - g0, n_tail = gend - gb;
        for (int rb = wave * 4; rb < n_head + n_tail; rb += 16) {
            const int x = rb + (lane >> 4);
            if (x < n_head + n_tail && c < D / 8) {
                const int r = x < n_head ? x : (gb - g0) + (x - n_head);
                const int jj = j0 + s_list[r];
                const size_t src = ((size_t)(row0 + jj) * v.Hkv + h) * D + c * 8;
                const uint4 kk = *reinterpret_cast<const uint4*>(k + src);
                const uint4 vl = *reinterpret_cast<const uint4*>(vv + src);
                const int gi = g0 + r;
                const int page = pt[gi >> 6];
                store_row_chunk<D>(pool_page(v, page), gi & 63, c, kk, vl);
                if (c == 0) {
                    v.pos_pool[(size_t)page * kPageTokens + (gi & 63)] = bi.T_old + jj;
                    v.logit_pool[(size_t)page * kPageTokens + (gi & 63)] = f[((size_t)row0 + jj) * v.Hkv + h];
                }
            }
        }
    }
}

hipError_t spkv_launch_append_bulk(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                                   const float* f, const SpkvCu& cu, int n_max, int32_t* prefix,
                                   hipStream_t s) {
    if (n_max <= v.w && n_max <= kSegTokens) {      // short chunks: one launch
        if (v.D == 128) spkv_bulk_ring<128, true, false><<<dim3(v.n_pairs), dim3(256), 0, s>>>(v, cu, prefix, k, vv, f);
        else spkv_bulk_ring<64, true, false><<<dim3(v.n_pairs), dim3(256), 0, s>>>(v, cu, prefix, k, vv, f);
        return hipGetLastError();
    }
    const int segs_all = (n_max + kSegTokens - 1) / kSegTokens;
    const int ring_blocks = (v.w + kHalfTokens - 1) / kHalfTokens;
    const dim3 grid3(segs_all + ring_blocks, v.n_pairs);
    const bool fold = segs_all <= kCountSegs;       // the per-pair launch counts for itself
    if (!fold) spkv_bulk_count<<<dim3(segs_all, v.n_pairs), dim3(256), 0, s>>>(v, f, cu);
    if (v.D == 128) {
        if (fold) spkv_bulk_ring<128, false, true><<<dim3(v.n_pairs), dim3(256), 0, s>>>(v, cu, prefix, k, vv, f);
        else spkv_bulk_ring<128, false, false><<<dim3(v.n_pairs), dim3(256), 0, s>>>(v, cu, prefix, k, vv, f);
        spkv_bulk_scatter<128><<<grid3, dim3(256), 0, s>>>(v, k, vv, f, cu, prefix, segs_all);
    } else {
        if (fold) spkv_bulk_ring<64, false, true><<<dim3(v.n_pairs), dim3(256), 0, s>>>(v, cu, prefix, k, vv, f);
        else spkv_bulk_ring<64, false, false><<<dim3(v.n_pairs), dim3(256), 0, s>>>(v, cu, prefix, k, vv, f);
        spkv_bulk_scatter<64><<<grid3, dim3(256), 0, s>>>(v, k, vv, f, cu, prefix, segs_all);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ prune after a raise
// After the threshold has been raised (Sec. 2.1: tau can be chosen after training, per
// deployment): every long-term entry whose stored logit no longer passes the gate is dropped
// and the list closed up, in place and in order.  One workgroup per (sequence, KV head)
// walks its list 256 entries at a time: flags, ranks by a block scan, then the kept rows
// move down 16 at a time -- read into registers, barrier, written.  A row's destination
// index never exceeds its own index and rows go in ascending order, so no write lands on a
// row that is still to be read.  Pages the shorter list no longer reaches go back onto the
// stack of recycled pages (pushes only: no page is allocated in this launch).
template <int D>
__global__ __launch_bounds__(256) void spkv_prune(SpkvView v) {
    const int pair = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, c = lane & 15;
    const int L = v.kept_len[pair];
    int32_t* pt = v.page_table + (size_t)pair * v.pt_cap;
    __shared__ int s_w[4];
    __shared__ uint16_t s_list[256];
    __shared__ int s_base;
    int out = 0;                                           // entries kept so far (uniform)
    for (int seg0 = 0; seg0 < L; seg0 += 256) {
        const int idx = seg0 + tid;
        bool keep = false;
        if (idx < L) {
            const size_t e = (size_t)pt[idx >> 6] * kPageTokens + (idx & 63);
            keep = gate_passes(v, v.logit_pool[e], v.pos_pool[e]);
        }
        int tot;
        const int rank = block_excl_scan(keep ? 1 : 0, s_w, tot);
        if (keep) s_list[rank] = (uint16_t)tid;
        __syncthreads();
        for (int rb = 0; rb < tot; rb += 16) {
            const int r = rb + wave * 4 + (lane >> 4);
            const bool mine = r < tot && c < D / 8;
            uint4 kk = {0u, 0u, 0u, 0u};
            unsigned w[4] = {0u, 0u, 0u, 0u};
            int pos = 0;
            float lg = 0.f;
            if (mine) {
                const int si = seg0 + s_list[r];
                const int sp_page = pt[si >> 6], sk = si & 63;
                const uint16_t* sp = pool_page(v, sp_page);
                kk = *reinterpret_cast<const uint4*>(sp + spkv_k_off(D, sk, c * 8));
                const uint16_t* vs = sp + spkv_v_off(D, sk, c * 8);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    w[e] = (unsigned)vs[(2 * e) * 8] | ((unsigned)vs[(2 * e + 1) * 8] << 16);
                pos = v.pos_pool[(size_t)sp_page * kPageTokens + sk];
                lg = v.logit_pool[(size_t)sp_page * kPageTokens + sk];
            }
            __syncthreads();                               // every row of the group has been read
            if (mine) {
                const int di = out + r;
                const int dp_page = pt[di >> 6], dk = di & 63;
                store_row_chunk<D>(pool_page(v, dp_page), dk, c, kk, make_uint4(w[0], w[1], w[2], w[3]));
                if (c == 0) {
                    v.pos_pool[(size_t)dp_page * kPageTokens + dk] = pos;
                    v.logit_pool[(size_t)dp_page * kPageTokens + dk] = lg;
                }
            }
            __syncthreads();                               // ... and written, before the next group reads
        }
        out += tot;
    }
    const int np_old = (L + kPageTokens - 1) / kPageTokens, np_new = (out + kPageTokens - 1) / kPageTokens;
    const int n_free = np_old - np_new;
    if (tid == 0) s_base = n_free > 0 ? atomicAdd(v.free_top, n_free) : 0;
    __syncthreads();
    for (int i = tid; i < n_free; i += 256) v.free_pages[s_base + i] = pt[np_new + i];
    if (tid == 0) v.kept_len[pair] = out;
}

hipError_t spkv_launch_prune(const SpkvView& v, hipStream_t s) {
    if (v.D == 128) spkv_prune<128><<<dim3(v.n_pairs), dim3(256), 0, s>>>(v);
    else spkv_prune<64><<<dim3(v.n_pairs), dim3(256), 0, s>>>(v);
    return hipGetLastError();
}

// ---------------------------------------------------------------- release a sequence
// One workgroup per KV head of the sequence: its pages go onto the stack of recycled pages
// and its counters back to zero (the ring needs no clearing: with T = 0 no slot is valid).
__global__ __launch_bounds__(256) void spkv_release_sequence(SpkvView v, int b) {
    const int pair = b * v.Hkv + blockIdx.x;
    const int tid = threadIdx.x;
    const int np = (v.kept_len[pair] + kPageTokens - 1) / kPageTokens;
    __shared__ int s_base;
    if (tid == 0) s_base = np > 0 ? atomicAdd(v.free_top, np) : 0;
    __syncthreads();
    for (int i = tid; i < np; i += 256)
        v.free_pages[s_base + i] = v.page_table[(size_t)pair * v.pt_cap + i];
    if (tid == 0) {
        v.kept_len[pair] = 0;
        v.t_pair[pair] = 0;
        v.gate_on[pair] = 0;
    }
}

hipError_t spkv_launch_release_sequence(const SpkvView& v, int b, hipStream_t s) {
    spkv_release_sequence<<<dim3(v.Hkv), dim3(256), 0, s>>>(v, b);
    return hipGetLastError();
}

// ------------------------------------------------------------ kept positions (debug)
__global__ __launch_bounds__(256) void spkv_gather_positions(SpkvView v, int pair) {
    const int L = v.kept_len[pair];
    for (int gi = blockIdx.x * blockDim.x + threadIdx.x; gi < L; gi += gridDim.x * blockDim.x) {
        const int page = v.page_table[(size_t)pair * v.pt_cap + (gi >> 6)];
        v.pos_scratch[gi] = v.pos_pool[(size_t)page * kPageTokens + (gi & 63)];
    }
}

hipError_t spkv_launch_gather_positions(const SpkvView& v, int pair, hipStream_t s) {
    spkv_gather_positions<<<dim3(64), dim3(256), 0, s>>>(v, pair);
    return hipGetLastError();
}

