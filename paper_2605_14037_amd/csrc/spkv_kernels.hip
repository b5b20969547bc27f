// HIP kernels of the SP-KV decode path for gfx950 (MI355X, wave64, MFMA).
//
//   write path : spkv_append_step (one token per sequence, fused evict + append),
//                spkv_bulk_count / spkv_bulk_ring / spkv_bulk_scatter (many tokens:
//                ballot + mbcnt stream compaction, stable order)
//   partition  : pair_split (every head's kept list cut into equal work items, derived
//                in both decode kernels from the device-side lengths)
//   read path  : spkv_decode_split (split-K flash decoding on MFMA, one wave per item),
//                spkv_decode_combine (log-sum-exp merge of the partials)
//   fused step : spkv_decode_split<.., true> + spkv_combine_append (append and decode of
//                one token per sequence in two launches instead of three)
//
// Gate: Eq. 2 of the paper taken on the logit, z = 1[f >= theta].  Availability:
// Eq. 3-4; the window ring holds exactly the keys with 0 <= t - s < w and the long-term
// pages exactly the gated-on keys with t - s >= w, so the two sets are disjoint and their
// union is the available set of Eq. 5.
#include <algorithm>

#include "spkv_internal.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) float f32x8;

#define SPKV_NEG_INF (-__builtin_inff())

// ------------------------------------------------------------------ small helpers
__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// 128-bit streaming load of 8 bf16.  K/V tiles are read once per decode step and never
// again before the whole cache has gone by, so they are loaded non-temporal: the lines
// bypass L2 / Infinity Cache retention instead of evicting the little that is reused
// (queries, page tables, partials).  Measured on MI355X: about 12 % more read bandwidth
// than plain loads for this access pattern.
__device__ __forceinline__ bf16x8 load_stream_b128(const uint16_t* p) {
    typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
    const u32x4 r = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return __builtin_bit_cast(bf16x8, r);
}

__device__ __forceinline__ int mbcnt64(unsigned long long mask) {
    return __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
}

__device__ __forceinline__ uint16_t* ring_page(const SpkvView& v, int pair, int rp) {
    return v.ring + ((size_t)pair * v.n_ring_pages + rp) * (size_t)spkv_page_elems(v.D);
}

__device__ __forceinline__ uint16_t* pool_page(const SpkvView& v, int page) {
    return v.pool + (size_t)page * (size_t)spkv_page_elems(v.D);
}

// The gate of the pair at position pos with utility logit f: Eq. 2 on the logit, or one of
// the first n_sink positions of the sequence (optional always-kept attention sinks, the
// "fixed attention sinks" variant of the ablations; n_sink = 0 is the paper's method).
__device__ __forceinline__ bool gate_passes(const SpkvView& v, float f, int pos) {
    return f >= v.theta || pos < v.n_sink;
}

// One pool page for the caller: a recycled one if the stack of released pages has any,
// else the next never-used one; -1 if the pool is exhausted.  Pushes onto the stack happen
// only in spkv_release_sequence, never in the same launch as pops, and a failed pop puts
// its decrement back, so the counter is exact between launches.
__device__ __forceinline__ int alloc_page(const SpkvView& v) {
    const int idx = atomicSub(v.free_top, 1) - 1;
    if (idx >= 0) return v.free_pages[idx];
    atomicAdd(v.free_top, 1);
    const int page = atomicAdd(v.pool_next, 1);
    return page < v.n_pages ? page : -1;
}

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

// ------------------------------------------------- write path, one token per sequence
// Appendix "Inference Kernels": write the new pair into the next ring slot; if the slot
// held a pair (window full), that pair leaves the window: keep it (append to the head's
// long-term pages, allocating a page with one atomic when a page boundary is crossed) if
// its stored logit passes the gate, else drop it.  One workgroup of D threads per
// (sequence, KV head); thread d moves V element d, threads < D/8 move one 16-byte K chunk.
// Append of one token to one (sequence, head), shared by spkv_append_step (workgroup of D
// threads) and spkv_combine_append (256 threads, the first D of them move data), in two
// halves so that a caller can put other work between the loads and the stores.
// `row` indexes the new token in k/vv/f; T and L are the pair's counters as read by every
// thread before any of them is updated.
template <int D>
struct AppendRegs {
    float f_old, f_new;
    int page_entry;
    uint16_t v_new, v_old;
    uint4 k_new, k_old;
};

// Everything the counters address, issued together (the outgoing row is read before it is
// known whether it is kept: 2 + 16 bytes per thread).
template <int D>
__device__ __forceinline__ AppendRegs<D> append_load(const SpkvView& v, int pair, int h, int row,
                                                     int T, int L, const uint16_t* __restrict__ k,
                                                     const uint16_t* __restrict__ vv,
                                                     const float* __restrict__ f, int tid) {
    AppendRegs<D> r;
    const bool mover = tid < D, kmover = tid < D / 8;
    const int slot = T % v.w;
    const uint16_t* rp = ring_page(v, pair, slot >> 6);
    const int rk = slot & 63;
    const bool full = T >= v.w;
    const int lp = L >> 6, gk = L & 63;
    const size_t src = ((size_t)row * v.Hkv + h) * D;
    r.f_old = full ? v.ring_logit[(size_t)pair * v.w + slot] : 0.f;
    r.page_entry = (gk != 0 && lp < v.pt_cap) ? v.page_table[(size_t)pair * v.pt_cap + lp] : -1;
    r.f_new = f[(size_t)row * v.Hkv + h];
    r.v_new = 0;
    r.v_old = 0;
    r.k_new = make_uint4(0u, 0u, 0u, 0u);
    r.k_old = make_uint4(0u, 0u, 0u, 0u);
    if (mover) r.v_new = vv[src + tid];
    if (kmover) r.k_new = *reinterpret_cast<const uint4*>(k + src + tid * 8);
    if (full) {
        if (mover) r.v_old = rp[spkv_v_off(D, rk, tid)];
        if (kmover) r.k_old = *reinterpret_cast<const uint4*>(rp + spkv_k_off(D, rk, tid * 8));
    }
    return r;
}

template <int D>
__device__ __forceinline__ void append_store(const SpkvView& v, int pair, int T, int L,
                                             const AppendRegs<D>& r, int tid, int* s_page) {
    const bool mover = tid < D, kmover = tid < D / 8;
    const int slot = T % v.w;
    uint16_t* rp = ring_page(v, pair, slot >> 6);
    const int rk = slot & 63;
    const bool full = T >= v.w;
    const int lp = L >> 6, gk = L & 63;
    const bool have_page = gk != 0 && lp < v.pt_cap;
    if (full && gate_passes(v, r.f_old, T - v.w)) {               // Eq. 2 on the logit
        int page = r.page_entry;
        if (!have_page) {                                         // first pair of a new page
            if (tid == 0) {
                const int np = lp < v.pt_cap ? alloc_page(v) : -1;
                if (np >= 0) v.page_table[(size_t)pair * v.pt_cap + lp] = np;
                else *v.err_flag = 1;
                *s_page = np;
            }
            __syncthreads();
            page = *s_page;
        }
        if (page >= 0) {
            uint16_t* gp = pool_page(v, page);
            if (mover) gp[spkv_v_off(D, gk, tid)] = r.v_old;
            if (kmover) *reinterpret_cast<uint4*>(gp + spkv_k_off(D, gk, tid * 8)) = r.k_old;
            if (tid == 0) {
                v.pos_pool[(size_t)page * kPageTokens + gk] = T - v.w;
                v.kept_len[pair] = L + 1;
            }
        }
    }
    if (mover) rp[spkv_v_off(D, rk, tid)] = r.v_new;
    if (kmover) *reinterpret_cast<uint4*>(rp + spkv_k_off(D, rk, tid * 8)) = r.k_new;
    if (tid == 0) {
        v.ring_logit[(size_t)pair * v.w + slot] = r.f_new;
        v.t_pair[pair] = T + 1;
        if (gate_passes(v, r.f_new, T)) v.gate_on[pair] += 1;
    }
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
    const AppendRegs<D> r = append_load<D>(v, pair, h, row, T, L, k, vv, f, threadIdx.x);
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
template <int D>
__global__ __launch_bounds__(256) void spkv_bulk_ring(SpkvView v, SpkvCu cu, int32_t* prefix) {
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

    // (a) how many ring pairs are kept
    int cnt = 0;
    for (int base = 0; base < nr; base += 256) {
        const int idx = base + tid;
        const bool flag = idx < nr && gate_passes(v, rl[(r0 + idx) % v.w], r0 + idx);
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
        const int nseg_all = (n + kSegTokens - 1) / kSegTokens;
        const int32_t* so = v.seg_on + (size_t)pair * v.n_seg_cap;
        int on = 0;
        for (int i = tid; i < nseg_all; i += 256) on += so[i];
        for (int o = 32; o > 0; o >>= 1) on += __shfl_xor(on, o);
        __syncthreads();
        if (lane == 0) s_w[wave] = on;
        __syncthreads();
        if (tid == 0) v.gate_on[pair] += s_w[0] + s_w[1] + s_w[2] + s_w[3];
    }

    // (c) pages: one allocation per new logical page, in parallel; the table entries are
    //     visible to the whole workgroup after the barrier and to stage 3 after the launch
    const int first = (L_old + kPageTokens - 1) / kPageTokens;
    const int last = (L_old + total_new + kPageTokens - 1) / kPageTokens;
    const int need = last <= v.pt_cap ? last - first : 0;
    int bad = last > v.pt_cap ? 1 : 0;
    for (int i = tid; i < need; i += 256) {
        const int page = alloc_page(v);
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
        const bool flag = idx < nr && gate_passes(v, rl[(r0 + idx) % v.w], r0 + idx);
        int tot;
        const int rank = block_excl_scan(flag ? 1 : 0, s_w, tot);
        if (flag) s_list[rank] = (uint16_t)tid;
        if (prefix != nullptr && idx < nr) {
            const int i = r0 + idx + v.w - T_old;      // the new token whose t - w is this position
            prefix[((size_t)cu.v[b] + i) * v.Hkv + (pair - b * v.Hkv)] = L_old + done + rank + (flag ? 1 : 0);
        }
        __syncthreads();
        const int c = lane & 15;
        for (int rb = wave * 4; rb < tot; rb += 16) {
            const int r = rb + (lane >> 4);
            if (r < tot && c < D / 8) {
                const int s = r0 + base + s_list[r];
                const int slot = s % v.w;
                const uint16_t* sp = ring_page(v, pair, slot >> 6);
                const int sk = slot & 63;
                const uint4 kk = *reinterpret_cast<const uint4*>(sp + spkv_k_off(D, sk, c * 8));
                const uint16_t* vs = sp + spkv_v_off(D, sk, c * 8);
                unsigned w[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    w[e] = (unsigned)vs[(2 * e) * 8] | ((unsigned)vs[(2 * e + 1) * 8] << 16);
                const int gi = L_old + done + r;
                const int page = pt[gi >> 6];
                store_row_chunk<D>(pool_page(v, page), gi & 63, c, kk, make_uint4(w[0], w[1], w[2], w[3]));
                if (c == 0) v.pos_pool[(size_t)page * kPageTokens + (gi & 63)] = s;
            }
        }
        done += tot;
        __syncthreads();
    }
}

// Stage 3: per (256-token segment, pair).  Thread i owns token j0 + i: gate flag, rank
// (mbcnt inside the wave + the popcounts of the lower waves + the segment offset from
// stage 2); the kept tokens' indices are compacted into LDS and their rows moved in groups
// of eight consecutive destination rows (whole 16-byte V units, transposed through LDS),
// stragglers row by row; the last min(n, w) tokens of the call are written into the ring.
template <int D>
__global__ __launch_bounds__(256) void spkv_bulk_scatter(SpkvView v, const uint16_t* __restrict__ k,
                                                         const uint16_t* __restrict__ vv,
                                                         const float* __restrict__ f, SpkvCu cu,
                                                         int32_t* prefix) {
    const int pair = blockIdx.y, seg = blockIdx.x;
    const int b = pair / v.Hkv, h = pair - b * v.Hkv;
    const int row0 = cu.v[b];
    const int n = cu.v[b + 1] - row0;
    const int j0 = seg * kSegTokens;
    if (j0 >= n) return;
    const BulkInfo bi = *reinterpret_cast<const BulkInfo*>(v.bulk_info + (size_t)pair * 8);
    if (bi.ok == 0) return;
    const int n_ev = max(0, n - v.w);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, c = lane & 15;
    __shared__ int s_cnt[4];
    __shared__ uint16_t s_list[256];
    __shared__ __attribute__((aligned(16))) uint16_t s_v[4][8][D];

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
            if (lane < 8)
                v.pos_pool[(size_t)page * kPageTokens + dk0 + lane] =
                    bi.T_old + j0 + s_list[G8 - g0 + lane];
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
                if (c == 0) v.pos_pool[(size_t)page * kPageTokens + (gi & 63)] = bi.T_old + jj;
            }
        }
    }
    const int ja = max(j0, n_ev), jb = min(n, j0 + kSegTokens);
    for (int rb = ja + wave * 4; rb < jb; rb += 16) {
        const int jj = rb + (lane >> 4);
        if (jj < jb && c < D / 8) {
            const int slot = (bi.T_old + jj) % v.w;
            const size_t src = ((size_t)(row0 + jj) * v.Hkv + h) * D + c * 8;
            const uint4 kk = *reinterpret_cast<const uint4*>(k + src);
            const uint4 vl = *reinterpret_cast<const uint4*>(vv + src);
            store_row_chunk<D>(ring_page(v, pair, slot >> 6), slot & 63, c, kk, vl);
            if (c == 0)
                v.ring_logit[(size_t)pair * v.w + slot] = f[((size_t)row0 + jj) * v.Hkv + h];
        }
    }
}

hipError_t spkv_launch_append_bulk(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                                   const float* f, const SpkvCu& cu, int n_max, int32_t* prefix,
                                   hipStream_t s) {
    const int segs_all = (n_max + kSegTokens - 1) / kSegTokens;
    spkv_bulk_count<<<dim3(segs_all, v.n_pairs), dim3(256), 0, s>>>(v, f, cu);
    if (v.D == 128) {
        spkv_bulk_ring<128><<<dim3(v.n_pairs), dim3(256), 0, s>>>(v, cu, prefix);
        spkv_bulk_scatter<128><<<dim3(segs_all, v.n_pairs), dim3(256), 0, s>>>(v, k, vv, f, cu, prefix);
    } else {
        spkv_bulk_ring<64><<<dim3(v.n_pairs), dim3(256), 0, s>>>(v, cu, prefix);
        spkv_bulk_scatter<64><<<dim3(segs_all, v.n_pairs), dim3(256), 0, s>>>(v, k, vv, f, cu, prefix);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ work partition
// Work unit: a half-page (32 keys).  Pair p has ceil(L/32) long-term half-pages followed
// by ceil(min(T, w)/32) ring half-pages.  The host picks hp_per_item (about total half-
// pages / target item count, from its upper bound of the lengths) and the slot count per
// pair; every pair is then cut evenly into ceil(n / hp_per_item) items from its exact
// device-side lengths, so that the split-K grid is balanced over the kept lengths
// whatever their spread.  Both decode kernels derive the same partition from (L, T).
struct PairSplit {
    int nhp;    // half-pages of the pair
    int ghp;    // of which long-term
    int items;  // work items the pair is cut into
    int L, T, Tw;
};

__device__ __forceinline__ PairSplit pair_split(const SpkvView& v, int pair, SpkvSplit sp) {
    PairSplit r;
    r.L = v.kept_len[pair];
    r.T = v.t_pair[pair];
    r.Tw = min(r.T, v.w);
    r.ghp = (r.L + kHalfTokens - 1) >> 5;
    r.nhp = r.ghp + ((r.Tw + kHalfTokens - 1) >> 5);
    r.items = min((r.nhp + sp.hp_per_item - 1) / sp.hp_per_item, sp.slots);
    return r;
}

// ------------------------------------------------------------------- split-K decode
// One half-page (32 keys) of flash decoding on the MFMA operands already in registers:
//   S[key][head]   = K[key][:] . Q[head][:]          2 x D/32 MFMA 16x16x32 (bf16 -> fp32)
//   online softmax in the log2 domain (running max m, sum l), weights rounded to bf16
//   O[d][head]    += V[key][d] * P[key][head]        D/16 MFMA 16x16x32
// Bit e of `kill` excludes this lane's key r = 8 kc + e (for the column this lane holds);
// `any_kill` is the wave-uniform "some lane has a bit set".
template <int D>
__device__ __forceinline__ void attend_half_page(const bf16x8 (&ka)[2][D / 32],
                                                 const bf16x8 (&va)[D / 16],
                                                 const bf16x8 (&qb)[D / 32], unsigned kill,
                                                 bool any_kill, float scale_log2e,
                                                 f32x4 (&acc)[D / 16], float& m, float& l) {
    constexpr int NS = D / 32, NB = D / 16;
    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int sl = 0; sl < NS; ++sl) {
        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[0][sl], qb[sl], s0, 0, 0, 0);
        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[1][sl], qb[sl], s1, 0, 0, 0);
    }
    // Lane (kc, n) now holds, for head n, the keys r = 8 kc + 4 t + i of the half-page.
    float x[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[i] = s0[i] * scale_log2e;
        x[4 + i] = s1[i] * scale_log2e;
    }
    if (any_kill) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if ((kill >> e) & 1u) x[e] = SPKV_NEG_INF;
    }
    float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])),
                     fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m, mx);
    // m_new is -inf only while every key seen so far was excluded; a finite reference then
    // keeps exp2(-inf - ref) = 0 instead of exp2(-inf + inf) = NaN.
    const float m_ref = (m_new == SPKV_NEG_INF) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m - m_ref);
    f32x8 p;
    float psum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        p[e] = __builtin_amdgcn_exp2f(x[e] - m_ref);
        psum += p[e];
    }
    l = l * alpha + psum;
    if (__ballot(m_new != m) != 0ull) {
#pragma unroll
        for (int db = 0; db < NB; ++db) acc[db] *= alpha;
    }
    m = m_new;
    const bf16x8 pb = __builtin_convertvector(p, bf16x8);
#pragma unroll
    for (int db = 0; db < NB; ++db)
        acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[db], pb, acc[db], 0, 0, 0);
}

// One wavefront per work item.  The G <= 16 query heads of the GQA group are the N = 16
// columns of every MFMA, so each K/V tile is read exactly once per group.  Every wave-wide
// load is 1 KB contiguous.
// Block id = pair * slots + j with an odd slot count: workgroups go round-robin to the 8
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
template <int D, bool FUSED>
__global__ __launch_bounds__(64) void spkv_decode_split(SpkvView v, const uint16_t* __restrict__ q,
                                                        float scale_log2e, SpkvSplit sp) {
    constexpr int NS = D / 32;   // head-dim slabs of one K tile
    constexpr int NB = D / 16;   // 16-wide output blocks
    const int pair = blockIdx.x / sp.slots;
    const int j = blockIdx.x - pair * sp.slots;
    const PairSplit ps = pair_split(v, pair, sp);
    if (FUSED && j == 0 && threadIdx.x == 0) v.pair_items[pair] = ps.items;
    if (j >= ps.items) return;
    const int hbase = ps.nhp / ps.items, hrem = ps.nhp - hbase * ps.items;
    const int hp0 = j * hbase + min(j, hrem);
    const int hp1 = hp0 + hbase + (j < hrem ? 1 : 0);
    const int b = pair / v.Hkv, h = pair - b * v.Hkv;
    const int lane = threadIdx.x, kc = lane >> 4, n = lane & 15;

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
    if (n < v.G) {
        const size_t slot = (size_t)pair * sp.slots + j;
        float* pa = v.part_acc + (slot * v.G + n) * D + kc * 4;
#pragma unroll
        for (int db = 0; db < NB; ++db) *reinterpret_cast<f32x4*>(pa + db * 16) = acc[db];
        if (kc == 0) {
            float* pm = v.part_ml + (slot * v.G + n) * 2;
            pm[0] = m;
            pm[1] = l;
        }
    }
}

// One wave folds the partials of one (pair, head) into a running (max, sum, acc) triple:
// with M the running max,  acc = sum_i 2^(m_i - M) acc_i,  den = sum_i 2^(m_i - M) l_i.
// The loads of successive items are independent; only the cheap rescaling is chained.
// Lane owns E = D / 64 output elements.
template <int D>
__device__ __forceinline__ void fold_items(const SpkvView& v, size_t slot0, int g, int first,
                                           int stride, int items, int lane, float& mw, float& den,
                                           float (&num)[D / 64]) {
    constexpr int E = D / 64;
    mw = SPKV_NEG_INF;
    den = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) num[e] = 0.f;
#pragma unroll 8
    for (int i = first; i < items; i += stride) {
        const float* pm = v.part_ml + ((slot0 + i) * v.G + g) * 2;
        const float* pa = v.part_acc + ((slot0 + i) * v.G + g) * D + lane * E;
        const float mi = pm[0], li = pm[1];
        float a[E];
#pragma unroll
        for (int e = 0; e < E; ++e) a[e] = pa[e];
        const float m_new = fmaxf(mw, mi);
        const float m_ref = (m_new == SPKV_NEG_INF) ? 0.f : m_new;   // items with no key: weight 0
        const float so = __builtin_amdgcn_exp2f(mw - m_ref), si = __builtin_amdgcn_exp2f(mi - m_ref);
        den = den * so + li * si;
#pragma unroll
        for (int e = 0; e < E; ++e) num[e] = num[e] * so + a[e] * si;
        mw = m_new;
    }
}

// Merge the partials of one (sequence, query head):
//   out = sum_i 2^(m_i - M) acc_i / sum_i 2^(m_i - M) l_i,  lse = (M + log2(sum)) ln 2.
// One workgroup of 4 waves per (pair, head): the waves take the items round-robin, each
// lane owns D/64 output elements, and the four wave results meet in LDS.
template <int D>
__global__ __launch_bounds__(256) void spkv_decode_combine(SpkvView v, uint16_t* __restrict__ out,
                                                           float* __restrict__ lse, SpkvSplit sp) {
    constexpr int E = D / 64;
    const int pair = blockIdx.x / v.G, g = blockIdx.x - pair * v.G;
    const int b = pair / v.Hkv, h = pair - b * v.Hkv;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int items = pair_split(v, pair, sp).items;
    const size_t slot0 = (size_t)pair * sp.slots;
    __shared__ float s_m[4];
    __shared__ float s_den[4];
    __shared__ float s_acc[4][D];

    float mw, den, num[E];
    fold_items<D>(v, slot0, g, wave, 4, items, lane, mw, den, num);
#pragma unroll
    for (int e = 0; e < E; ++e) s_acc[wave][lane * E + e] = num[e];
    if (lane == 0) {
        s_m[wave] = mw;
        s_den[wave] = den;
    }
    __syncthreads();
    if (tid < D) {
        const float M = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
        float nsum = 0.f, dsum = 0.f;
#pragma unroll
        for (int wv = 0; wv < 4; ++wv) {
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
// v_new); the workgroup of the group's first head then performs the append of the new
// token exactly as spkv_append_step does.  The item
// count of the pair comes from pair_items (written by the split kernel), not from the
// counters, so the other heads' workgroups never read what the append is changing.
template <int D>
__global__ __launch_bounds__(256) void spkv_combine_append(SpkvView v, uint16_t* __restrict__ out,
                                                           float* __restrict__ lse, SpkvSplit sp,
                                                           const uint16_t* __restrict__ k_new,
                                                           const uint16_t* __restrict__ v_new,
                                                           const float* __restrict__ f_new,
                                                           const uint16_t* __restrict__ q,
                                                           float scale_log2e) {
    constexpr int E = D / 64;
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
    __shared__ float s_m[4];
    __shared__ float s_den[4];
    __shared__ float s_acc[4][D];
    __shared__ int s_page;
    // The append's loads are issued before the merge and consumed after it.
    int T = 0, L = 0;
    AppendRegs<D> ar;
    if (g == 0) {
        T = v.t_pair[pair];
        L = v.kept_len[pair];
        ar = append_load<D>(v, pair, h, b, T, L, k_new, v_new, f_new, tid);
    }

    float mw, den, num[E];
    fold_items<D>(v, slot0, g, wave, 4, items, lane, mw, den, num);
#pragma unroll
    for (int e = 0; e < E; ++e) s_acc[wave][lane * E + e] = num[e];
    if (lane == 0) {
        s_m[wave] = mw;
        s_den[wave] = den;
    }
    __syncthreads();
    if (tid < D) {
        const float M = fmaxf(fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3])), m_tok);
        const float w_tok = __builtin_amdgcn_exp2f(m_tok - M);
        const unsigned ve = v_new[kv_row + tid];
        float nsum = __builtin_bit_cast(float, ve << 16) * w_tok, dsum = w_tok;
#pragma unroll
        for (int wv = 0; wv < 4; ++wv) {
            const float sc = __builtin_amdgcn_exp2f(s_m[wv] - M);
            nsum += s_acc[wv][tid] * sc;
            dsum += s_den[wv] * sc;
        }
        const size_t o = ((size_t)b * v.Hq + (size_t)h * v.G + g);
        const __bf16 r = (__bf16)(nsum / dsum);
        out[o * D + tid] = __builtin_bit_cast(uint16_t, r);
        if (lse != nullptr && tid == 0) lse[o] = (M + log2f(dsum)) * 0.6931471805599453f;
    }
    if (g == 0) append_store<D>(v, pair, T, L, ar, tid, &s_page);
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
//      (sequence, KV head) -- 32 MFMA columns (token, head) in two groups of 16 -- walks
//      the long-term prefix and then the staging rows of the block's windows, one online
//      softmax per column, and writes the normalised bf16 rows.  No partials, no combine.
// Window keys and long-term entries are disjoint (positions > t - w against <= t - w), so
// every available key is counted once.

struct SpkvPrefill {
    uint16_t* stage;     // [n_pairs][shp] half-pages
    int32_t*  prefix;    // [total tokens][H_kv]
    float*    bias;      // soft gating only: [n_pairs][shp][32] log2 u of every staging row
    int32_t   shp;       // staging half-pages per pair
    int32_t   tb;        // tokens per wave (32 / G)
    int32_t   nblk;      // workgroups (spans of 8 tb tokens) per pair in the grid
    int32_t   pin_xcd;   // 1: all blocks of a pair run on one XCD (shared L2)
};

// Eight V rows held in LDS (s_rows[row][d]) leave as 16-byte units: eight consecutive keys
// of one head-dim element, rows dk0 .. dk0 + 7 of page (or half-page) dp.  Lanes < D / 2.
template <int D>
__device__ __forceinline__ void store_v_units(uint16_t* dp, int dk0, const uint16_t (*s_rows)[D],
                                              int lane) {
    if (lane < D / 2) {
        unsigned dw[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) dw[r] = *reinterpret_cast<const unsigned*>(&s_rows[r][2 * lane]);
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
}

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
constexpr int kPrefillGroups = 2;    // column groups of 16 per wave
constexpr int kPrefillWaves = 8;     // waves per workgroup (two per SIMD)

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

// One workgroup of kPrefillWaves = 8 waves per span of 8 * tb consecutive tokens of one
// (sequence, KV head); wave wv owns tokens i0 = span start + wv * tb .. + tb - 1 as its
// 32 MFMA columns (tb = 32 / G tokens times G heads, two groups of 16).  The waves walk the
// same half-pages, so each 16 KB tile is fetched from memory once per workgroup into an LDS
// double buffer (every wave copies an eighth of the next tile while all consume the current
// one) and each wave reads its MFMA A operands from LDS with conflict-free 16-byte reads;
// 256 query columns share one tile fetch.  With 32 columns a wave needs about 200 VGPRs and
// no accumulation registers, so two waves fit a SIMD and one wave's vector work (weights)
// can run beside the other's MFMAs.  (Measured alternatives: four waves of 64 columns, one
// per SIMD, 15 % slower -- every latency is exposed; the same with the tile loop software-
// pipelined by hand, slower still; issue priority for one wave of each SIMD, 27 % slower.)
template <int D, bool SOFT>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void spkv_prefill_attend(SpkvView v, const uint16_t* __restrict__ q,
                                                           uint16_t* __restrict__ out,
                                                           float* __restrict__ lse, float scale_log2e,
                                                           SpkvPrefill pf, SpkvCu cu) {
    constexpr int NS = D / 32, NB = D / 16, NQ = kPrefillGroups, NW = kPrefillWaves;
    constexpr int kHalfElems = 2 * kHalfTokens * D;
    constexpr int kRows = kHalfElems / 512;     // 1 KB rows of a tile
    constexpr int kRowsPerWave = kRows / NW;
    __shared__ __attribute__((aligned(16))) uint16_t s_tile[2][kHalfElems];
    int pair, qblk;
    if (pf.pin_xcd) {
        // workgroups go round-robin to the 8 XCDs: id % 8 picks the XCD, and every pair
        // lives on XCD pair % 8, so its list is fetched into one L2 and re-read there
        const int local = blockIdx.x >> 3, lp = local / pf.nblk;
        qblk = local - lp * pf.nblk;
        // rotate inside every full group of 8 pairs by the group index: with 8 KV heads a
        // plain pair % 8 would give each XCD one head of every sequence, and heads differ
        // several-fold in kept length
        const int rot = (lp * 8 + 8 <= v.n_pairs) ? lp : 0;
        pair = lp * 8 + (((blockIdx.x & 7) + rot) & 7);
        if (pair >= v.n_pairs) return;
    } else {
        pair = blockIdx.x / pf.nblk;
        qblk = blockIdx.x - pair * pf.nblk;
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

    const int32_t* pt = v.page_table + (size_t)pair * v.pt_cap;
    const uint16_t* stage = pf.stage + (size_t)pair * pf.shp * (size_t)kHalfElems;
    auto base_of = [&](int x) -> const uint16_t* {
        x = min(x, last);
        if (x < nA) {
            const int page = min(max(pt[min(x >> 1, v.pt_cap - 1)], 0), v.n_pages - 1);
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

    const int my_off = (wv * kRowsPerWave * 64 + lane) * 8;     // this lane's part of a tile
    typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
    u32x4 t[kRowsPerWave];
    {
        const uint16_t* p = base_of(0) + my_off;
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r) t[r] = *reinterpret_cast<const u32x4*>(p + r * 512);
#pragma unroll
        for (int r = 0; r < kRowsPerWave; ++r)
            *reinterpret_cast<u32x4*>(&s_tile[0][my_off + r * 512]) = t[r];
    }
    const uint16_t* p_next = base_of(1);
    __syncthreads();

    // Tile loop.  The inner loop never touches the accumulators except by MFMA; when the
    // references do not fit a tile the wave leaves it before using the tile, rescales, and
    // resumes at the same tile (prefetch and barrier of a tile are issued exactly once, so
    // the waves stay in step whatever each one does).  After a rescale the references
    // are at least the tile's column maxima, so the second attempt is accepted; a column
    // with every key excluded so far keeps m = -inf and is accepted on the retry as well.
    int x = 0;
    bool resume = false, pending = false;
    float xs[NQ][8];
    while (x < n_hp) {
        if (pending) rescale_columns<D, NQ>(xs, SOFT ? 1.0f : scale_log2e, acc, m, l);
        for (; x < n_hp; ++x) {
            if (!resume) {
                // next tile (after the last one: the same tile again, into the idle buffer)
                const uint16_t* p = p_next + my_off;
#pragma unroll
                for (int r = 0; r < kRowsPerWave; ++r) t[r] = *reinterpret_cast<const u32x4*>(p + r * 512);
                p_next = base_of(x + 2);
            }
            resume = false;
            const uint16_t* tile = s_tile[x & 1];
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
                    const float4* bp = reinterpret_cast<const float4*>(
                        pf.bias + ((size_t)pair * pf.shp + (u_tile >> 5)) * kHalfTokens + kc * 8);
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
#pragma unroll
            for (int r = 0; r < kRowsPerWave; ++r)
                *reinterpret_cast<u32x4*>(&s_tile[(x + 1) & 1][my_off + r * 512]) = t[r];
            __syncthreads();
        }
    }

#pragma unroll
    for (int c = 0; c < NQ; ++c) {
        float lc = l[c];
        lc += __shfl_xor(lc, 16);
        lc += __shfl_xor(lc, 32);
        if (tok[c] >= 0) {
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

static SpkvPrefill prefill_params(const SpkvView& v, int n_max, uint16_t* stage, int32_t* prefix,
                                  float* bias, int shp) {
    SpkvPrefill pf;
    pf.stage = stage;
    pf.prefix = prefix;
    pf.bias = bias;
    pf.shp = shp;
    pf.tb = (16 * kPrefillGroups) / v.G;
    pf.nblk = (n_max + kPrefillWaves * pf.tb - 1) / (kPrefillWaves * pf.tb);   // spans of one workgroup
    pf.pin_xcd = (v.n_pairs >= 8 && pf.nblk >= 4) ? 1 : 0;
    return pf;
}

static unsigned prefill_grid(const SpkvView& v, const SpkvPrefill& pf) {
    return pf.pin_xcd ? 8u * (unsigned)((v.n_pairs + 7) / 8) * (unsigned)pf.nblk
                      : (unsigned)v.n_pairs * (unsigned)pf.nblk;
}

hipError_t spkv_launch_prefill(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                               const float* f, const uint16_t* q, uint16_t* out, float* lse,
                               float sm_scale, const SpkvCu& cu, int n_max, uint16_t* stage,
                               int32_t* prefix, int shp, hipStream_t s) {
    const SpkvPrefill pf = prefill_params(v, n_max, stage, prefix, nullptr, shp);
    const float sl = sm_scale * 1.4426950408889634f;
    const int stage_hps = (v.w + n_max + kHalfTokens - 1) / kHalfTokens;
    const unsigned grid = prefill_grid(v, pf);
    hipError_t e;
    if (v.D == 128) {
        spkv_prefill_stage<128><<<dim3(stage_hps, v.n_pairs), dim3(256), 0, s>>>(v, k, vv, f, cu, pf);
        if ((e = spkv_launch_append_bulk(v, k, vv, f, cu, n_max, prefix, s)) != hipSuccess) return e;
        spkv_prefill_attend<128, false><<<dim3(grid), dim3(64 * kPrefillWaves), 0, s>>>(v, q, out, lse, sl, pf, cu);
    } else {
        spkv_prefill_stage<64><<<dim3(stage_hps, v.n_pairs), dim3(256), 0, s>>>(v, k, vv, f, cu, pf);
        if ((e = spkv_launch_append_bulk(v, k, vv, f, cu, n_max, prefix, s)) != hipSuccess) return e;
        spkv_prefill_attend<64, false><<<dim3(grid), dim3(64 * kPrefillWaves), 0, s>>>(v, q, out, lse, sl, pf, cu);
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
        spkv_prefill_attend<128, true><<<dim3(grid), dim3(64 * kPrefillWaves), 0, s>>>(v, q, out, lse, sl, pf, cu);
    } else {
        spkv_prefill_stage<64><<<dim3(stage_hps, v.n_pairs), dim3(256), 0, s>>>(v, k, vv, f, cu, pf);
        spkv_prefill_attend<64, true><<<dim3(grid), dim3(64 * kPrefillWaves), 0, s>>>(v, q, out, lse, sl, pf, cu);
    }
    return hipGetLastError();
}

hipError_t spkv_launch_decode(const SpkvView& v, const uint16_t* q, uint16_t* out, float* lse,
                              float sm_scale, SpkvSplit sp, bool split_only, hipEvent_t ev0,
                              hipEvent_t ev1, hipStream_t s) {
    const float scale_log2e = sm_scale * 1.4426950408889634f;
    const unsigned grid = (unsigned)v.n_pairs * (unsigned)sp.slots;
    hipError_t e;
    if (ev0 != nullptr && (e = hipEventRecord(ev0, s)) != hipSuccess) return e;
    if (v.D == 128)
        spkv_decode_split<128, false><<<dim3(grid), dim3(64), 0, s>>>(v, q, scale_log2e, sp);
    else
        spkv_decode_split<64, false><<<dim3(grid), dim3(64), 0, s>>>(v, q, scale_log2e, sp);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (ev1 != nullptr && (e = hipEventRecord(ev1, s)) != hipSuccess) return e;
    if (split_only) return hipSuccess;
    if (v.D == 128)
        spkv_decode_combine<128><<<dim3(v.n_pairs * v.G), dim3(256), 0, s>>>(v, out, lse, sp);
    else
        spkv_decode_combine<64><<<dim3(v.n_pairs * v.G), dim3(256), 0, s>>>(v, out, lse, sp);
    return hipGetLastError();
}

int spkv_split_resident_items(int head_dim) {
    int dev = 0, cus = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    const hipError_t e =
        head_dim == 128
            ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, spkv_decode_split<128, false>, 64, 0)
            : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, spkv_decode_split<64, false>, 64, 0);
    if (e != hipSuccess || per_cu <= 0 || cus <= 0) return 0;
    return per_cu * cus;
}

hipError_t spkv_launch_decode_step(const SpkvView& v, const uint16_t* k, const uint16_t* vv,
                                   const float* f, const uint16_t* q, uint16_t* out, float* lse,
                                   float sm_scale, SpkvSplit sp, hipStream_t s) {
    const float scale_log2e = sm_scale * 1.4426950408889634f;
    const unsigned grid = (unsigned)v.n_pairs * (unsigned)sp.slots;
    if (v.D == 128) {
        spkv_decode_split<128, true><<<dim3(grid), dim3(64), 0, s>>>(v, q, scale_log2e, sp);
        spkv_combine_append<128><<<dim3(v.n_pairs * v.G), dim3(256), 0, s>>>(v, out, lse, sp, k, vv, f, q, scale_log2e);
    } else {
        spkv_decode_split<64, true><<<dim3(grid), dim3(64), 0, s>>>(v, q, scale_log2e, sp);
        spkv_combine_append<64><<<dim3(v.n_pairs * v.G), dim3(256), 0, s>>>(v, out, lse, sp, k, vv, f, q, scale_log2e);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ utility predictor
// Eq. 1 with the predictor of the paper's listing: Linear(d_model, d_hidden) - SiLU -
// Linear(d_hidden, n_kv_heads), pre-sigmoid.  Hidden layer: one workgroup per (16 hidden
// units, 16 tokens); its four waves split d_model, each running MFMA 16x16x32 with the W1
// rows as A operand (rows = hidden units, contraction over d_model) and the tokens as the
// 16 columns; partial sums meet in LDS, bias and SiLU are applied in fp32.
__global__ __launch_bounds__(256) void spkv_predictor_hidden(const uint16_t* __restrict__ x,
                                                             const uint16_t* __restrict__ w1,
                                                             const float* __restrict__ b1,
                                                             float* __restrict__ act, int n_tokens,
                                                             int d_model, int d_hidden) {
    const int j0 = blockIdx.x * 16, t0 = blockIdx.y * 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, kc = lane >> 4, n = lane & 15;
    const int kq = d_model / 4;                       // this wave's share of d_model
    const uint16_t* wrow = w1 + (size_t)(j0 + n) * d_model + wave * kq + kc * 8;
    const bool tok_ok = t0 + n < n_tokens;
    const uint16_t* xrow = x + (size_t)(tok_ok ? t0 + n : 0) * d_model + wave * kq + kc * 8;
    // (columns past the last token read token 0's row; their results are never stored)
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int k = 0; k < kq; k += 32) {            // kq is a multiple of 32 (d_model of 128)
        const uint4 a = *reinterpret_cast<const uint4*>(wrow + k);
        const uint4 bv = *reinterpret_cast<const uint4*>(xrow + k);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                      __builtin_bit_cast(bf16x8, bv), acc, 0, 0, 0);
    }
    // lane (kc, n) holds hidden units j0 + 4 kc + i of token t0 + n
    __shared__ float s_part[4][16][17];
#pragma unroll
    for (int i = 0; i < 4; ++i) s_part[wave][4 * kc + i][n] = acc[i];
    __syncthreads();
    const int jj = tid >> 4, tt = tid & 15;
    if (t0 + tt < n_tokens) {
        float h = s_part[0][jj][tt] + s_part[1][jj][tt] + s_part[2][jj][tt] + s_part[3][jj][tt];
        if (b1 != nullptr) h += b1[j0 + jj];
        act[(size_t)(t0 + tt) * d_hidden + j0 + jj] = h / (1.f + __expf(-h));     // SiLU
    }
}

// Output layer: one wave per (token, KV head): logits = b2 + W2[h, :] . act[t, :].
__global__ __launch_bounds__(64) void spkv_predictor_out(const float* __restrict__ act,
                                                         const uint16_t* __restrict__ w2,
                                                         const float* __restrict__ b2,
                                                         float* __restrict__ logits, int d_hidden,
                                                         int n_kv_heads) {
    const int t = blockIdx.x / n_kv_heads, h = blockIdx.x - t * n_kv_heads;
    float sum = 0.f;
    for (int j = threadIdx.x; j < d_hidden; j += 64) {
        const unsigned wbits = w2[(size_t)h * d_hidden + j];
        sum += __builtin_bit_cast(float, wbits << 16) * act[(size_t)t * d_hidden + j];
    }
    for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
    if (threadIdx.x == 0) logits[(size_t)t * n_kv_heads + h] = sum + (b2 != nullptr ? b2[h] : 0.f);
}

hipError_t spkv_launch_predictor(const uint16_t* x, const uint16_t* w1, const float* b1,
                                 const uint16_t* w2, const float* b2, float* logits, float* act,
                                 int n_tokens, int d_model, int d_hidden, int n_kv_heads,
                                 hipStream_t s) {
    spkv_predictor_hidden<<<dim3(d_hidden / 16, (n_tokens + 15) / 16), dim3(256), 0, s>>>(
        x, w1, b1, act, n_tokens, d_model, d_hidden);
    spkv_predictor_out<<<dim3(n_tokens * n_kv_heads), dim3(64), 0, s>>>(act, w2, b2, logits, d_hidden,
                                                                        n_kv_heads);
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
