// Device-side helpers shared by the kernel files: vector types, streaming loads, page
// addressing, the gate, page allocation, the single-token append (used by the write kernel
// and by the fused decode step), the work partition and one half-page of flash decoding on
// MFMA operands held in registers.
#pragma once
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

// Stores that other compute dies (each has its own L2) may read later in the SAME launch:
// written through to device scope, so that waiting for the wave's outstanding stores is all
// it takes to make them visible -- no write-back of the whole L2 (a device-scope release fence
// costs that, and thousands of them per launch were measured at +200 us).
// (The s_nop: a store of more than 8 bytes reads its data registers up to two cycles after it
// issues, and the compiler, which keeps that distance for its own stores, does not look into
// an asm statement -- without it the next instruction may overwrite the data.)
__device__ __forceinline__ void store_device_b128(float* p, f32x4 x) {
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 1" : : "v"(p), "v"(x) : "memory");
}
__device__ __forceinline__ void store_device_b32(float* p, float x) {
    __hip_atomic_store(p, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Waits for every vector memory operation of this wave, the stores above included.
__device__ __forceinline__ void wait_all_vmem() { asm volatile("s_waitcnt vmcnt(0)" : : : "memory"); }

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

// `need` pages at once, for one thread of a workgroup that then hands them out: one atomic on
// the bump counter (and one on the stack of recycled pages only when it holds any) instead of
// one or three per page -- every atomic of a launch goes to the same two addresses, and they
// are served one after the other.  Page i of the batch: batch_page(v, pb, i); -1 past the pool.
struct PageBatch {
    int stack_lo, from_stack, pool_base;
};
__device__ __forceinline__ PageBatch alloc_page_batch(const SpkvView& v, int need) {
    PageBatch pb = {0, 0, 0};
    if (need <= 0) return pb;
    // no page is pushed in a launch that pops, so a stack seen empty stays empty
    if (__hip_atomic_load(v.free_top, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) > 0) {
        const int top = atomicSub(v.free_top, need);
        const int take = min(max(top, 0), need);
        if (take < need) atomicAdd(v.free_top, need - take);     // put back what was not there
        pb.from_stack = take;
        pb.stack_lo = top - take;
    }
    const int rest = need - pb.from_stack;
    if (rest > 0) pb.pool_base = atomicAdd(v.pool_next, rest);
    return pb;
}
__device__ __forceinline__ int batch_page(const SpkvView& v, const PageBatch& pb, int i) {
    if (i < pb.from_stack) return v.free_pages[pb.stack_lo + i];
    const int page = pb.pool_base + (i - pb.from_stack);
    return page < v.n_pages ? page : -1;
}

// ------------------------------------------------------------------ memory -> LDS copies
// One wave-wide 16-byte load from global memory straight into LDS: lane i's 16 bytes at
// `src` land at LDS byte address lds_row + 16 i (lds_row wave-uniform).  The load counts
// as a vector memory load in flight until its data is in LDS.  (No memory clobber: the
// compiler would then stop treating the page table as read-only and turn its scalar lookups
// into vector loads that wait for these copies.  What orders the copies against the LDS
// reads is the workgroup barrier, which neither the asm nor the reads may cross.)
__device__ __forceinline__ void load_row_to_lds(const uint16_t* src, unsigned lds_row) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(src), "s"(lds_row)
                 : "m0");
}

// The same for one dword per lane: lane i's 4 bytes land at lds_row + 4 i.
__device__ __forceinline__ void load_word_to_lds(const float* src, unsigned lds_row) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
                 :
                 : "v"(src), "s"(lds_row)
                 : "m0");
}

// Waits until at most N of this wave's vector memory loads are still in flight (they
// complete in the order issued).
template <int N>
__device__ __forceinline__ void wait_loads_but() {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N));
}

// ------------------------------------------------------------------ utility predictor
// Hidden layer of the predictor (Eq. 1) for 16 hidden units x 16 tokens over kq (a multiple
// of 32) elements of d_model: lane (kc, n) passes its row of W1 (unit n) and of the tokens'
// hidden states (token n), both offset by kc * 8 elements; it gets the sums of units
// 4 kc .. 4 kc + 3 for token n.  Loads go out eight steps at a time so that the memory
// round trips overlap (the tail repeats the last step's loads and skips its MFMAs).
__device__ __forceinline__ f32x4 predictor_contract(const uint16_t* __restrict__ wrow,
                                                    const uint16_t* __restrict__ xrow, int kq) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < kq; k0 += 256) {
        uint4 a[8], bv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int k = min(k0 + u * 32, kq - 32);
            a[u] = *reinterpret_cast<const uint4*>(wrow + k);
            bv[u] = *reinterpret_cast<const uint4*>(xrow + k);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (k0 + u * 32 < kq)
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[u]),
                                                              __builtin_bit_cast(bf16x8, bv[u]),
                                                              acc, 0, 0, 0);
    }
    return acc;
}

// ------------------------------------------------- write path, one token per sequence
// Appendix "Inference Kernels": write the new pair into the next ring slot; if the slot
// held a pair (window full), that pair leaves the window: keep it (append to the head's
// long-term pages, allocating a page with one atomic when a page boundary is crossed) if
// its stored logit passes the gate, else drop it.  One workgroup of D threads per
// (sequence, KV head); thread d moves V element d, threads < D/8 move one 16-byte K chunk.
// Append of one token to one (sequence, head), shared by spkv_append_step (workgroup of D
// threads) and spkv_combine_append (256 or 1024 threads, the first D of them move data), in two
// halves so that a caller can put other work between the loads and the stores.
// `row` indexes the new token in k/vv, f_new is its logit for this head; T and L are the
// pair's counters as read by every thread before any of them is updated.
// NT = threads that take part (a multiple of 64); thread tid moves V elements tid,
// tid + NT, ... (one per thread when NT >= D).
template <int D, int NT = D>
struct AppendRegs {
    static constexpr int VPT = (D + NT - 1) / NT;
    float f_old, f_new;
    int page_entry;
    uint16_t v_new[VPT], v_old[VPT];
    uint4 k_new, k_old;
};

// Everything the counters address, issued together (the outgoing row is read before it is
// known whether it is kept: 2 + 16 bytes per thread).
template <int D, int NT = D>
__device__ __forceinline__ AppendRegs<D, NT> append_load(const SpkvView& v, int pair, int h, int row,
                                                         int T, int L, const uint16_t* __restrict__ k,
                                                         const uint16_t* __restrict__ vv,
                                                         float f_new, int tid) {
    AppendRegs<D, NT> r;
    constexpr int VPT = AppendRegs<D, NT>::VPT;
    const bool kmover = tid < D / 8;
    const int slot = T % v.w;
    const uint16_t* rp = ring_page(v, pair, slot >> 6);
    const int rk = slot & 63;
    const bool full = T >= v.w;
    const int lp = L >> 6, gk = L & 63;
    const size_t src = ((size_t)row * v.Hkv + h) * D;
    r.f_old = full ? v.ring_logit[(size_t)pair * v.w + slot] : 0.f;
    r.page_entry = (gk != 0 && lp < v.pt_cap) ? v.page_table[(size_t)pair * v.pt_cap + lp] : -1;
    r.f_new = f_new;
    r.k_new = make_uint4(0u, 0u, 0u, 0u);
    r.k_old = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        const int d = tid + j * NT;
        r.v_new[j] = 0;
        r.v_old[j] = 0;
        if (d < D) {
            r.v_new[j] = vv[src + d];
            if (full) r.v_old[j] = rp[spkv_v_off(D, rk, d)];
        }
    }
    if (kmover) {
        r.k_new = *reinterpret_cast<const uint4*>(k + src + tid * 8);
        if (full) r.k_old = *reinterpret_cast<const uint4*>(rp + spkv_k_off(D, rk, tid * 8));
    }
    return r;
}

template <int D, int NT = D>
__device__ __forceinline__ void append_store(const SpkvView& v, int pair, int T, int L,
                                             const AppendRegs<D, NT>& r, int tid, int* s_page) {
    constexpr int VPT = AppendRegs<D, NT>::VPT;
    const bool kmover = tid < D / 8;
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
#pragma unroll
            for (int j = 0; j < VPT; ++j) {
                const int d = tid + j * NT;
                if (d < D) gp[spkv_v_off(D, gk, d)] = r.v_old[j];
            }
            if (kmover) *reinterpret_cast<uint4*>(gp + spkv_k_off(D, gk, tid * 8)) = r.k_old;
            if (tid == 0) {
                v.pos_pool[(size_t)page * kPageTokens + gk] = T - v.w;
                v.logit_pool[(size_t)page * kPageTokens + gk] = r.f_old;
                v.kept_len[pair] = L + 1;
            }
        }
    }
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
        const int d = tid + j * NT;
        if (d < D) rp[spkv_v_off(D, rk, d)] = r.v_new[j];
    }
    if (kmover) *reinterpret_cast<uint4*>(rp + spkv_k_off(D, rk, tid * 8)) = r.k_new;
    if (tid == 0) {
        v.ring_logit[(size_t)pair * v.w + slot] = r.f_new;
        v.t_pair[pair] = T + 1;
        if (gate_passes(v, r.f_new, T)) v.gate_on[pair] += 1;
    }
}

// ------------------------------------------------------------------ work partition
// Work unit: a half-page (32 keys).  Pair p has ceil(L/32) long-term half-pages followed
// by ceil(min(T, w)/32) ring half-pages.  The host picks hp_per_item (about total half-
// pages / target item count, from its upper bound of the lengths) and the slot count per
// pair; every pair is then cut evenly into ceil(n / hp_per_item) items from its exact
// device-side lengths, so that the split-K grid is balanced over the kept lengths
// whatever their spread.  Both decode kernels derive the same partition from (L, T).
//
// With sp.mw > 1 (single-token decode kernels only) mw one-wave items share a workgroup and
// merge their results there: the pair gets min(ceil(n / (mw hp_per_item)), slots) workgroups,
// one partial slot each, and is cut evenly into min(groups * mw, n) items.
struct PairSplit {
    int nhp;    // half-pages of the pair
    int ghp;    // of which long-term
    int groups; // partial slots in use (= items for mw = 1)
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
    const int per = sp.hp_per_item * sp.mw;
    r.groups = min((r.nhp + per - 1) / per, sp.slots);
    r.items = min(r.groups * sp.mw, r.nhp);
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

