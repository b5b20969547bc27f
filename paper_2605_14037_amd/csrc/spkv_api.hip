// Host side of the SP-KV C ABI: configuration checks, arena carving, the host's
// conservative capacity bound (the "safe budget" idea of the paper's appendix "Inference
// Kernels": capacity is checked on the host without reading the device until a worst-case
// bound trips), and kernel launches.  See include/spkv.h for the contract.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "spkv_internal.h"

namespace {

constexpr size_t kAlign = 256;
constexpr int kFallbackItems = 2944;   // 11.5 one-wave workgroups per CU on 256 CUs (MI355X, 12 fit)
constexpr int kMaxTimedLaunches = 8192;

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Carve {
    size_t ring, ring_logit, t_pair, kept_len, gate_on, pool_next, free_top, free_pages, err_flag,
        page_table, pool,
        pos_pool, logit_pool, seg_count, seg_on, bulk_info, part_acc, part_ml, pair_items,
        pair_ticket, pos_scratch, chunk_stage, chunk_prefix, total;
    int n_pairs, G, n_ring_pages, pt_cap, n_pages, n_seg_cap, max_items, chunk_shp;
};

bool config_ok(const spkv_config_t* c) {
    if (c == nullptr) return false;
    if (c->batch < 1 || c->batch > SPKV_MAX_BATCH) return false;
    if (c->n_kv_heads < 1 || c->n_q_heads < 1 || c->n_q_heads % c->n_kv_heads != 0) return false;
    if (c->n_q_heads / c->n_kv_heads > 16) return false;
    if ((int64_t)c->batch * c->n_kv_heads > 16384) return false;
    if (c->head_dim != 64 && c->head_dim != 128) return false;
    if (c->window < 1 || c->window > (1 << 20)) return false;
    if (c->page_tokens != 0 && c->page_tokens != SPKV_PAGE_TOKENS) return false;
    if (std::isnan(c->tau)) return false;
    if (c->max_context < 1 || c->max_context > (1 << 30)) return false;
    if (c->max_total_kept_tokens < 0 || c->max_total_kept_tokens > ((int64_t)1 << 40)) return false;
    return true;
}

bool carve(const spkv_config_t* c, Carve* out) {
    if (!config_ok(c)) return false;
    Carve k{};
    k.n_pairs = c->batch * c->n_kv_heads;
    k.G = c->n_q_heads / c->n_kv_heads;
    k.n_ring_pages = (c->window + kPageTokens - 1) / kPageTokens;
    const int64_t max_evicted = c->max_context > c->window ? c->max_context - c->window : 0;
    k.pt_cap = (int)((max_evicted + kPageTokens - 1) / kPageTokens) + 1;
    const int64_t n_pages = (c->max_total_kept_tokens + kPageTokens - 1) / kPageTokens + k.n_pairs;
    if (n_pages > ((int64_t)1 << 30)) return false;
    k.n_pages = (int)n_pages;
    k.n_seg_cap = (int)(((int64_t)c->max_context + kSegTokens - 1) / kSegTokens) + 1;
    // Work-item slots: 128 per pair leaves room for a pair 40 times longer than the mean at
    // the default item count; at least enough for the largest item target on one pair.
    // The multi-token kernels store 16, 32 or 64 columns per slot instead of G: two slots of
    // 64 columns per pair must fit whatever the shape (only caches of thousands of pairs
    // with small groups reach this term).
    k.max_items = std::max(kMaxItemTarget + k.n_pairs, std::min(k.n_pairs * 128, 1 << 17));
    k.max_items = std::max(k.max_items, (k.n_pairs * 128 + k.G - 1) / k.G);
    const size_t page_bytes = (size_t)spkv_page_elems(c->head_dim) * 2;
    size_t off = 0;
    auto take = [&off](size_t bytes) {
        const size_t at = off;
        off += align_up(bytes);
        return at;
    };
    k.ring = take((size_t)k.n_pairs * k.n_ring_pages * page_bytes);
    k.ring_logit = take((size_t)k.n_pairs * c->window * 4);
    k.t_pair = take((size_t)k.n_pairs * 4);
    k.kept_len = take((size_t)k.n_pairs * 4);
    k.gate_on = take((size_t)k.n_pairs * 4);
    k.pool_next = take(4);
    k.free_top = take(4);
    k.free_pages = take((size_t)k.n_pages * 4);
    k.err_flag = take(4);
    k.page_table = take((size_t)k.n_pairs * k.pt_cap * 4);
    k.pool = take((size_t)k.n_pages * page_bytes);
    k.pos_pool = take((size_t)k.n_pages * kPageTokens * 4);
    k.logit_pool = take((size_t)k.n_pages * kPageTokens * 4);
    k.seg_count = take((size_t)k.n_pairs * k.n_seg_cap * 4);
    k.seg_on = take((size_t)k.n_pairs * k.n_seg_cap * 4);
    k.bulk_info = take((size_t)k.n_pairs * 32);
    k.part_acc = take((size_t)k.max_items * k.G * c->head_dim * 4);
    k.part_ml = take((size_t)k.max_items * k.G * 2 * 4);
    k.pair_items = take((size_t)k.n_pairs * 4);
    k.pair_ticket = take((size_t)k.n_pairs * 4);
    k.pos_scratch = take((size_t)k.pt_cap * kPageTokens * 4);
    // multi-token steps (spkv_decode_chunk) wider than one group of 16 query columns run on the
    // prefill kernels: staging half-pages for the window plus 16 new rows per pair, and the
    // per-token prefix counts
    k.chunk_shp = (int)(((int64_t)c->window + SPKV_MAX_CHUNK_TOKENS + kHalfTokens - 1) / kHalfTokens);
    k.chunk_stage = take((size_t)k.n_pairs * k.chunk_shp * ((size_t)2 * kHalfTokens * c->head_dim * 2));
    k.chunk_prefix = take((size_t)c->batch * SPKV_MAX_CHUNK_TOKENS * c->n_kv_heads * 4);
    k.total = off;
    *out = k;
    return true;
}

float logit_threshold(float tau) {
    const double t = (double)tau;
    if (t <= 0.0) return -INFINITY;
    if (t >= 1.0) return INFINITY;
    return (float)std::log(t / (1.0 - t));
}

int64_t pages_for(int64_t len) { return (len + kPageTokens - 1) / kPageTokens; }

}  // namespace

// Scratch for spkv_decode_attention_static: the split-K partials of callers that cannot
// allocate.  One copy per GPU the library runs on, held until the process ends.  In host
// code the array's name is only a handle for hipGetSymbolAddress; kernels get the address
// that call returns for the current device.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of the current device's copy of `scratch` (looked up once per device);
// null if the runtime cannot tell.
void* static_scratch_of_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

struct spkv_cache {
    spkv_config_t cfg;
    Carve carve;
    SpkvView view;
    char* arena;
    size_t arena_bytes;
    std::vector<int32_t> T;       // tokens per sequence (exact: the host sees every append)
    std::vector<int32_t> L_ub;    // per (seq, head): upper bound of the long-term length
    int64_t pages_ub;             // sum of pages_for(L_ub): upper bound of pool pages in use
    bool bound_is_loose;          // a bulk append grew L_ub by far more than the truth
    // Single-token steps add one to L_ub per pair and step although only the keep rate's share
    // is kept, so the bound drifts away from the lengths and the work partition derived from
    // it would come out too coarse.  `slack` counts what was added since the bound was last
    // exact; past 1/16 of the bound the lengths are copied to pinned host memory behind the
    // step just issued (no wait) and adopted by the first later call that finds the copy done.
    int64_t slack;
    int32_t* snap_host;           // pinned, [n_pairs]; null if the allocation failed
    hipEvent_t snap_event;
    bool snap_pending;
    std::vector<int32_t> snap_ev; // per sequence: pairs pushed out of the window since the copy
    int item_target;
    int merge_waves;              // SPKV_OPT_MERGE_WAVES (0 = per call)
    int step_launches;            // SPKV_OPT_STEP_LAUNCHES (0 = per call)
    int n_sink;                   // always-kept first positions (SPKV_OPT_SINK_TOKENS)
    int one_round_items;          // items the chip runs in one resident round, with a margin
    int chunk_round_items[3];     // the same for the chunk kernel with 1, 2, 4 column groups
    SpkvSplit split;              // partition used by the last decode call
    bool timing;
    bool split_only;
    std::vector<hipEvent_t> events;   // pairs (before, after)
    int n_timed;
};

namespace {

// Point the device-side view at the regions of the cache's arena.
void bind_view(spkv_cache* c) {
    const spkv_config_t* cfg = &c->cfg;
    const Carve& k = c->carve;
    SpkvView& v = c->view;
    v.B = cfg->batch;
    v.Hq = cfg->n_q_heads;
    v.Hkv = cfg->n_kv_heads;
    v.G = k.G;
    v.D = cfg->head_dim;
    v.w = cfg->window;
    v.n_pairs = k.n_pairs;
    v.n_ring_pages = k.n_ring_pages;
    v.pt_cap = k.pt_cap;
    v.n_pages = k.n_pages;
    v.n_seg_cap = k.n_seg_cap;
    v.max_items = k.max_items;
    v.theta = logit_threshold(cfg->tau);
    v.n_sink = c->n_sink;
    char* a = c->arena;
    v.ring = reinterpret_cast<uint16_t*>(a + k.ring);
    v.ring_logit = reinterpret_cast<float*>(a + k.ring_logit);
    v.t_pair = reinterpret_cast<int32_t*>(a + k.t_pair);
    v.kept_len = reinterpret_cast<int32_t*>(a + k.kept_len);
    v.gate_on = reinterpret_cast<int32_t*>(a + k.gate_on);
    v.pool_next = reinterpret_cast<int32_t*>(a + k.pool_next);
    v.free_top = reinterpret_cast<int32_t*>(a + k.free_top);
    v.free_pages = reinterpret_cast<int32_t*>(a + k.free_pages);
    v.err_flag = reinterpret_cast<int32_t*>(a + k.err_flag);
    v.page_table = reinterpret_cast<int32_t*>(a + k.page_table);
    v.pool = reinterpret_cast<uint16_t*>(a + k.pool);
    v.pos_pool = reinterpret_cast<int32_t*>(a + k.pos_pool);
    v.logit_pool = reinterpret_cast<float*>(a + k.logit_pool);
    v.seg_count = reinterpret_cast<int32_t*>(a + k.seg_count);
    v.seg_on = reinterpret_cast<int32_t*>(a + k.seg_on);
    v.bulk_info = reinterpret_cast<int32_t*>(a + k.bulk_info);
    v.part_acc = reinterpret_cast<float*>(a + k.part_acc);
    v.part_ml = reinterpret_cast<float*>(a + k.part_ml);
    v.pair_items = reinterpret_cast<int32_t*>(a + k.pair_items);
    v.pair_ticket = reinterpret_cast<int32_t*>(a + k.pair_ticket);
    v.pos_scratch = reinterpret_cast<int32_t*>(a + k.pos_scratch);
}

// Read the exact long-term lengths back and tighten the host's bound.  Synchronises.
int refresh_bound(spkv_cache* c, hipStream_t s, int32_t* kept_len_out) {
    std::vector<int32_t> len(c->carve.n_pairs);
    if (hipStreamSynchronize(s) != hipSuccess) return SPKV_E_HIP;
    if (hipMemcpy(len.data(), c->view.kept_len, len.size() * 4, hipMemcpyDeviceToHost) != hipSuccess)
        return SPKV_E_HIP;
    int64_t pages = 0;
    for (int p = 0; p < c->carve.n_pairs; ++p) {
        c->L_ub[p] = len[p];
        pages += pages_for(len[p]);
    }
    c->pages_ub = pages;
    c->bound_is_loose = false;
    c->slack = 0;
    c->snap_pending = false;      // a copy still on its way is older than what was just read
    if (kept_len_out != nullptr) std::memcpy(kept_len_out, len.data(), len.size() * 4);
    return SPKV_OK;
}

// Keeps the host's bound of the lengths close to the truth during long runs of single-token
// steps without ever waiting: adopts a finished copy of the device lengths (plus whatever has
// left the windows since it was enqueued: still an upper bound), and enqueues a new copy when
// the slack has grown past 1/16 of the bound.  Never while the stream is being captured (the
// copy would become a graph node and the host would read it at the wrong time).
void tighten_bound(spkv_cache* c, hipStream_t s) {
    if (c->snap_host == nullptr) return;
    const int n_pairs = c->carve.n_pairs, Hkv = c->cfg.n_kv_heads;
    if (c->snap_pending) {
        const hipError_t q = hipEventQuery(c->snap_event);
        if (q == hipSuccess) {
            int64_t pages = 0, slack = 0;
            for (int p = 0; p < n_pairs; ++p) {
                const int64_t L = (int64_t)c->snap_host[p] + c->snap_ev[p / Hkv];
                if (L < c->L_ub[p]) c->L_ub[p] = (int32_t)L;
                pages += pages_for(c->L_ub[p]);
                slack += c->snap_ev[p / Hkv];
            }
            c->pages_ub = pages;
            c->slack = slack;
            c->snap_pending = false;
        } else {
            (void)hipGetLastError();      // "not ready" is not an error of the next launch
            return;
        }
    }
    int64_t sum = 0;
    for (int p = 0; p < n_pairs; ++p) sum += c->L_ub[p] + std::min(c->T[p / Hkv], c->cfg.window);
    if (c->slack * 16 <= sum) return;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(s, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) {
        (void)hipGetLastError();
        return;
    }
    if (hipMemcpyAsync(c->snap_host, c->view.kept_len, (size_t)n_pairs * 4, hipMemcpyDeviceToHost, s) !=
            hipSuccess ||
        hipEventRecord(c->snap_event, s) != hipSuccess) {
        (void)hipGetLastError();
        return;
    }
    std::fill(c->snap_ev.begin(), c->snap_ev.end(), 0);
    c->snap_pending = true;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Work partition for one decode call from the host's upper bound of the lengths: items of
// about (all half-pages / item_target) half-pages, and enough slots per pair for the
// longest pair.  The kernels apply it to the exact device-side lengths, which never
// exceed the bound, so every pair fits its slots.
// mw: work items per workgroup and partial slot; the target counts items either way.
SpkvSplit choose_split_mw(const spkv_cache* c, int one_round_items, int64_t slots_total_cap, int mw,
                          int64_t* n_items = nullptr) {
    const int n_pairs = c->carve.n_pairs, Hkv = c->cfg.n_kv_heads;
    std::vector<int64_t> hp(n_pairs);
    int64_t sum_hp = 0, max_hp = 1;
    for (int p = 0; p < n_pairs; ++p) {
        const int Tw = std::min(c->T[p / Hkv], c->cfg.window);
        hp[p] = (c->L_ub[p] + kHalfTokens - 1) / kHalfTokens + (Tw + kHalfTokens - 1) / kHalfTokens;
        sum_hp += hp[p];
        max_hp = std::max(max_hp, hp[p]);
    }
    // Item count: the caller's target, else one resident round, whatever the cache size and
    // however the pairs differ in length -- every pair is cut evenly, so no item is longer
    // than the others.  (Measured: more, shorter items cost 6 % on a batch of 64 sequences
    // of 1k-64k tokens with keep rates from 0 to 1, 2.9 GB kept, and 11 % on 2.1 GB in 128
    // equal lists: every item pays its own start-up round trips.)
    int64_t target = c->item_target;
    if (target <= 0) target = one_round_items;
    target = std::max<int64_t>(1, std::min<int64_t>(target, slots_total_cap - n_pairs));
    const int64_t groups_target = std::max<int64_t>(1, target / mw);
    int64_t per = std::max<int64_t>(1, (sum_hp + groups_target * mw - 1) / (groups_target * mw));
    // Every pair rounds its workgroup count up; keep the total within the target, because one
    // more than the chip holds at once costs a whole second round of the longest items.
    for (int guard = 0; guard < 64; ++guard) {
        int64_t groups = 0;
        for (int p = 0; p < n_pairs; ++p) groups += (hp[p] + per * mw - 1) / (per * mw);
        if (groups <= groups_target || groups <= n_pairs) break;
        per += std::max<int64_t>(1, per / 16);
    }
    const int64_t slots_cap = std::max<int64_t>(1, slots_total_cap / n_pairs - 1);
    if ((max_hp + per * mw - 1) / (per * mw) > slots_cap) per = (max_hp + slots_cap * mw - 1) / (slots_cap * mw);
    SpkvSplit sp;
    sp.hp_per_item = (int32_t)per;
    sp.slots = (int32_t)((max_hp + per * mw - 1) / (per * mw)) | 1;   // odd: see spkv_decode_split
    sp.mw = mw;
    if (n_items != nullptr) {
        *n_items = 0;
        for (int p = 0; p < n_pairs; ++p)
            *n_items += std::min<int64_t>((hp[p] + per * mw - 1) / (per * mw) * mw, hp[p]);
    }
    return sp;
}

// Single-token decode: workgroups of 4 or 2 items when the cache has few pairs and the
// whole-workgroup rounding per pair neither lengthens the items nor leaves fewer of them than
// one item per workgroup would.  Measured (step time, 32 query / 8 KV heads of 128, keep rates
// drawn per pair): one sequence of 128k tokens 26 -> 22 us, 4 of 128k 39 -> 38, 3 of 64k
// 47 -> 44, equal lists of 1 to 4 sequences 1 to 2.5 us less, two of twelve shapes 1.5 us
// more; but 16 sequences of 32k (128 pairs of about 23 items) 78 -> 92 at the same item
// length, and 64 sequences of 1k-64k 459 -> 540: workgroup ids go round-robin to the 8 XCDs,
// pair p's run starts at id p * slots, and when the lengths repeat from sequence to sequence
// (keep rates that depend on the head) every sequence adds the same uneven pattern -- in
// units of whole workgroups -- until some XCD is handed more waves than it holds and runs
// the surplus in a second round.  Hence the limit of kMergePairs pairs.
constexpr int kMergePairs = 32;
SpkvSplit choose_split(const spkv_cache* c, int one_round_items, int64_t slots_total_cap) {
    int64_t items_one = 0;
    const SpkvSplit one = choose_split_mw(c, one_round_items, slots_total_cap, 1, &items_one);
    if (c->merge_waves == 1) return one;
    if (c->merge_waves > 1) return choose_split_mw(c, one_round_items, slots_total_cap, c->merge_waves);
    if (c->carve.n_pairs > kMergePairs) return one;
    for (int mw = 4; mw > 1; mw >>= 1) {
        int64_t items = 0;
        const SpkvSplit sp = choose_split_mw(c, one_round_items, slots_total_cap, mw, &items);
        if (sp.hp_per_item <= one.hp_per_item && items >= items_one) return sp;
    }
    return one;
}

SpkvSplit choose_split(const spkv_cache* c) {
    return choose_split(c, c->one_round_items, c->carve.max_items);
}

// One launch (merge and append by the last workgroup of every pair) or two (a merge launch)
// for the single-token decode calls.
// Measured on MI355X (16 sequences, 32 query / 8 KV heads of 128, step time in us against kept
// K/V bytes): one launch 22.3 / 36.8 / 54.6 / 87.3 at 51 / 115 / 222 / 436 MB, two launches
// 17.6 / 28.0 / 45.0 / 78.5 -- the tickets (an atomic per workgroup on one address per pair,
// served one after the other) and the merge's dependent round trips inside the launch cost
// more than a second launch does, at every size tried.  Two launches unless the caller asks.
bool one_launch(const spkv_cache* c, hipStream_t) {
    return c->step_launches == 1;
}

// Tokens sequence b receives in a call: from cu_seqlens, or one each (cu == nullptr).
int tokens_for(const int32_t* cu, int b) { return cu == nullptr ? 1 : cu[b + 1] - cu[b]; }

// Capacity check before any launch.  Worst case for the pool: every pair pushed out of
// the window by this call is kept.  If that does not fit, the true lengths are read back
// once (synchronises) and the check repeated; SPKV_E_CAPACITY if it still does not fit.
int reserve_capacity(spkv_cache* c, const int32_t* cu, hipStream_t s) {
    const int B = c->cfg.batch, Hkv = c->cfg.n_kv_heads, w = c->cfg.window;
    for (int b = 0; b < B; ++b)
        if ((int64_t)c->T[b] + tokens_for(cu, b) > c->cfg.max_context) return SPKV_E_CAPACITY;
    for (int attempt = 0;; ++attempt) {
        int64_t pages = c->pages_ub;
        for (int b = 0; b < B; ++b) {
            const int n = tokens_for(cu, b);
            const int64_t ev = std::max<int64_t>(0, (int64_t)c->T[b] + n - w) -
                               std::max<int64_t>(0, (int64_t)c->T[b] - w);
            if (ev == 0) continue;
            for (int h = 0; h < Hkv; ++h) {
                const int64_t L = c->L_ub[b * Hkv + h];
                pages += pages_for(L + ev) - pages_for(L);
            }
        }
        if (pages <= c->carve.n_pages) return SPKV_OK;
        if (attempt == 1) return SPKV_E_CAPACITY;
        const int rc = refresh_bound(c, s, nullptr);
        if (rc != SPKV_OK) return rc;
    }
}

// Host bookkeeping after the launch: exact token counts, upper bounds of the lengths.
void commit_lengths(spkv_cache* c, const int32_t* cu) {
    const int B = c->cfg.batch, Hkv = c->cfg.n_kv_heads, w = c->cfg.window;
    for (int b = 0; b < B; ++b) {
        const int n = tokens_for(cu, b);
        const int64_t ev = std::max<int64_t>(0, (int64_t)c->T[b] + n - w) -
                           std::max<int64_t>(0, (int64_t)c->T[b] - w);
        c->T[b] += n;
        if (ev == 0) continue;
        for (int h = 0; h < Hkv; ++h) {
            int32_t& L = c->L_ub[b * Hkv + h];
            c->pages_ub += pages_for(L + ev) - pages_for(L);
            L += (int32_t)ev;
        }
        c->slack += ev * Hkv;
        c->snap_ev[b] += (int32_t)ev;
    }
}

}  // namespace

extern "C" {

size_t spkv_cache_required_bytes(const spkv_config_t* cfg) {
    Carve k;
    return carve(cfg, &k) ? k.total : 0;
}

int spkv_cache_create(const spkv_config_t* cfg, void* dev_arena, size_t arena_bytes, void* stream,
                      spkv_cache_t** out) {
    if (out == nullptr) return SPKV_E_INVAL;
    *out = nullptr;
    Carve k;
    if (!carve(cfg, &k)) return SPKV_E_INVAL;
    if (dev_arena == nullptr || (reinterpret_cast<uintptr_t>(dev_arena) % kAlign) != 0 ||
        arena_bytes < k.total)
        return SPKV_E_INVAL;
    spkv_cache* c = new (std::nothrow) spkv_cache();
    if (c == nullptr) return SPKV_E_NOMEM;
    c->cfg = *cfg;
    c->cfg.page_tokens = SPKV_PAGE_TOKENS;
    c->carve = k;
    c->arena = static_cast<char*>(dev_arena);
    c->arena_bytes = k.total;
    c->T.assign(cfg->batch, 0);
    c->L_ub.assign(k.n_pairs, 0);
    c->pages_ub = 0;
    c->bound_is_loose = false;
    c->slack = 0;
    c->snap_host = nullptr;
    c->snap_event = nullptr;
    c->snap_pending = false;
    c->snap_ev.assign(cfg->batch, 0);
    c->item_target = 0;
    c->merge_waves = 0;
    c->step_launches = 0;
    c->n_sink = 0;
    {
        // Measured on MI355X: up to 94 % of the resident slots run in one round; at 99 % some
        // compute units already queue a second item and the launch takes 15-20 % longer.
        const int resident = spkv_split_resident_items(cfg->head_dim);
        c->one_round_items = resident > 0 ? resident - resident / 24 : kFallbackItems;
        c->chunk_round_items[0] = c->chunk_round_items[1] = c->chunk_round_items[2] = 0;
    }
    c->split = SpkvSplit{1, 1, 1};
    c->timing = false;
    c->split_only = false;
    c->n_timed = 0;
    bind_view(c);
    if (spkv_launch_fill_zero(c->arena, c->arena_bytes, static_cast<hipStream_t>(stream)) !=
        hipSuccess) {
        delete c;
        return SPKV_E_HIP;
    }
    (void)static_scratch_of_current_device();     // set-up for spkv_decode_attention_static
    // pinned host buffer for the length snapshots (see tighten_bound); the cache works
    // without it, with a coarser partition on very long generations
    void* pinned = nullptr;
    if (hipHostMalloc(&pinned, (size_t)k.n_pairs * 4, hipHostMallocDefault) == hipSuccess &&
        hipEventCreateWithFlags(&c->snap_event, hipEventDisableTiming) == hipSuccess) {
        c->snap_host = static_cast<int32_t*>(pinned);
    } else {
        if (pinned != nullptr) (void)hipHostFree(pinned);
        c->snap_event = nullptr;
        (void)hipGetLastError();
    }
    *out = c;
    return SPKV_OK;
}

int spkv_cache_grow(spkv_cache_t* c, const spkv_config_t* cfg, void* dev_arena, size_t arena_bytes,
                    void* stream) {
    if (c == nullptr || cfg == nullptr) return SPKV_E_INVAL;
    const spkv_config_t& o = c->cfg;
    if (cfg->batch != o.batch || cfg->n_q_heads != o.n_q_heads || cfg->n_kv_heads != o.n_kv_heads ||
        cfg->head_dim != o.head_dim || cfg->window != o.window)
        return SPKV_E_INVAL;
    if (cfg->max_context < o.max_context || cfg->max_total_kept_tokens < o.max_total_kept_tokens)
        return SPKV_E_INVAL;
    Carve k;
    if (!carve(cfg, &k)) return SPKV_E_INVAL;
    char* na = static_cast<char*>(dev_arena);
    if (na == nullptr || (reinterpret_cast<uintptr_t>(na) % kAlign) != 0 || arena_bytes < k.total)
        return SPKV_E_INVAL;
    // the two arenas must not overlap
    if (na < c->arena + c->arena_bytes && c->arena < na + k.total) return SPKV_E_INVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Carve& q = c->carve;
    const size_t page_bytes = (size_t)spkv_page_elems(o.head_dim) * 2;
    if (spkv_launch_fill_zero(na, k.total, s) != hipSuccess) return SPKV_E_HIP;
    struct Region { size_t to, from, bytes; };
    const Region regions[] = {
        {k.ring, q.ring, (size_t)q.n_pairs * q.n_ring_pages * page_bytes},
        {k.ring_logit, q.ring_logit, (size_t)q.n_pairs * o.window * 4},
        {k.t_pair, q.t_pair, (size_t)q.n_pairs * 4},
        {k.kept_len, q.kept_len, (size_t)q.n_pairs * 4},
        {k.gate_on, q.gate_on, (size_t)q.n_pairs * 4},
        {k.pool_next, q.pool_next, 4},
        {k.free_top, q.free_top, 4},
        {k.free_pages, q.free_pages, (size_t)q.n_pages * 4},
        {k.err_flag, q.err_flag, 4},
        {k.pool, q.pool, (size_t)q.n_pages * page_bytes},
        {k.pos_pool, q.pos_pool, (size_t)q.n_pages * kPageTokens * 4},
        {k.logit_pool, q.logit_pool, (size_t)q.n_pages * kPageTokens * 4},
    };
    // every region starts on a 256-byte boundary and is padded to one, and no region
    // shrinks, so copying the padded size stays inside the new region
    for (const Region& r : regions)
        if (spkv_launch_copy(na + r.to, c->arena + r.from, align_up(r.bytes), s) != hipSuccess)
            return SPKV_E_HIP;
    if (spkv_launch_copy_rows(reinterpret_cast<int32_t*>(na + k.page_table),
                              reinterpret_cast<const int32_t*>(c->arena + q.page_table), q.n_pairs,
                              q.pt_cap, k.pt_cap, s) != hipSuccess)
        return SPKV_E_HIP;
    const float tau = c->cfg.tau;
    c->cfg = *cfg;
    c->cfg.page_tokens = SPKV_PAGE_TOKENS;
    c->cfg.tau = tau;                    // the live threshold stays (see spkv_cache_set_tau)
    c->carve = k;
    c->arena = na;
    c->arena_bytes = k.total;
    bind_view(c);
    return SPKV_OK;
}

int spkv_cache_destroy(spkv_cache_t* c) {
    if (c == nullptr) return SPKV_E_INVAL;
    for (hipEvent_t e : c->events) (void)hipEventDestroy(e);
    if (c->snap_host != nullptr) {
        (void)hipEventSynchronize(c->snap_event);      // a copy may still be writing the buffer
        (void)hipEventDestroy(c->snap_event);
        (void)hipHostFree(c->snap_host);
    }
    delete c;
    return SPKV_OK;
}

int spkv_cache_reset(spkv_cache_t* c, void* stream) {
    if (c == nullptr) return SPKV_E_INVAL;
    if (spkv_launch_fill_zero(c->arena, c->arena_bytes, static_cast<hipStream_t>(stream)) != hipSuccess)
        return SPKV_E_HIP;
    std::fill(c->T.begin(), c->T.end(), 0);
    std::fill(c->L_ub.begin(), c->L_ub.end(), 0);
    c->pages_ub = 0;
    c->bound_is_loose = false;
    c->slack = 0;
    c->snap_pending = false;
    return SPKV_OK;
}

int spkv_append(spkv_cache_t* c, const void* k, const void* v, const float* util_logits,
                const int32_t* cu_seqlens, void* stream) {
    if (c == nullptr || cu_seqlens == nullptr) return SPKV_E_INVAL;
    const int B = c->cfg.batch;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (cu_seqlens[0] != 0) return SPKV_E_INVAL;
    int n_max = 0;
    for (int b = 0; b < B; ++b) {
        const int64_t n = (int64_t)cu_seqlens[b + 1] - cu_seqlens[b];
        if (n < 0) return SPKV_E_INVAL;
        if (n > n_max) n_max = (int)std::min<int64_t>(n, INT32_MAX);
    }
    if (n_max == 0) return SPKV_OK;
    if (k == nullptr || v == nullptr || util_logits == nullptr) return SPKV_E_INVAL;
    if (!aligned16(k) || !aligned16(v) || !aligned16(util_logits)) return SPKV_E_INVAL;
    const int rc = reserve_capacity(c, cu_seqlens, s);
    if (rc != SPKV_OK) return rc;

    SpkvCu cu;
    std::memcpy(cu.v, cu_seqlens, (size_t)(B + 1) * 4);
    const uint16_t* kk = static_cast<const uint16_t*>(k);
    const uint16_t* vv = static_cast<const uint16_t*>(v);
    hipError_t e = (n_max == 1)
                       ? spkv_launch_append_step(c->view, kk, vv, util_logits, cu, s)
                       : spkv_launch_append_bulk(c->view, kk, vv, util_logits, cu, n_max, nullptr, s);
    if (e != hipSuccess) return SPKV_E_HIP;
    commit_lengths(c, cu_seqlens);
    if (n_max > SPKV_MAX_CHUNK_TOKENS) c->bound_is_loose = true;   // short chunks: see tighten_bound
    return SPKV_OK;
}

int spkv_decode_step(spkv_cache_t* c, const void* k, const void* v, const float* util_logits,
                     const void* q, void* out, float* lse, float sm_scale, void* stream) {
    if (c == nullptr || k == nullptr || v == nullptr || util_logits == nullptr || q == nullptr ||
        out == nullptr)
        return SPKV_E_INVAL;
    if (!aligned16(k) || !aligned16(v) || !aligned16(util_logits) || !aligned16(q) ||
        !aligned16(out) || (lse != nullptr && !aligned16(lse)))
        return SPKV_E_INVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!(sm_scale > 0.f)) sm_scale = 1.0f / std::sqrt((float)c->cfg.head_dim);
    if (c->bound_is_loose) {
        const int rc = refresh_bound(c, s, nullptr);
        if (rc != SPKV_OK) return rc;
    }
    tighten_bound(c, s);
    const int rc = reserve_capacity(c, nullptr, s);
    if (rc != SPKV_OK) return rc;
    c->split = choose_split(c);          // partition of the state BEFORE the append
    if (spkv_launch_decode_step(c->view, static_cast<const uint16_t*>(k),
                                static_cast<const uint16_t*>(v), util_logits,
                                static_cast<const uint16_t*>(q), static_cast<uint16_t*>(out), lse,
                                sm_scale, c->split, one_launch(c, s), s) != hipSuccess)
        return SPKV_E_HIP;
    commit_lengths(c, nullptr);
    return SPKV_OK;
}

size_t spkv_decode_step_predict_workspace_bytes(int32_t batch, int32_t d_hidden) {
    if (batch <= 0 || d_hidden <= 0) return 0;
    return (size_t)kPredictSplit * batch * d_hidden * sizeof(float);
}

int spkv_decode_step_predict(spkv_cache_t* c, const void* hidden, const void* w1, const float* b1,
                             const void* w2, const float* b2, int32_t d_model, int32_t d_hidden,
                             const void* k, const void* v, const void* q, void* out, float* lse,
                             float* util_logits, void* workspace, size_t workspace_bytes,
                             float sm_scale, void* stream) {
    if (c == nullptr || hidden == nullptr || w1 == nullptr || w2 == nullptr || k == nullptr ||
        v == nullptr || q == nullptr || out == nullptr || util_logits == nullptr || workspace == nullptr)
        return SPKV_E_INVAL;
    if (d_model <= 0 || d_model % 128 != 0 || d_hidden <= 0 || d_hidden % 16 != 0) return SPKV_E_INVAL;
    if (!aligned16(hidden) || !aligned16(w1) || !aligned16(w2) || !aligned16(k) || !aligned16(v) ||
        !aligned16(q) || !aligned16(out) || !aligned16(util_logits) || !aligned16(workspace) ||
        (b1 != nullptr && !aligned16(b1)) || (b2 != nullptr && !aligned16(b2)) ||
        (lse != nullptr && !aligned16(lse)))
        return SPKV_E_INVAL;
    if (workspace_bytes < spkv_decode_step_predict_workspace_bytes(c->cfg.batch, d_hidden))
        return SPKV_E_INVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!(sm_scale > 0.f)) sm_scale = 1.0f / std::sqrt((float)c->cfg.head_dim);
    if (c->bound_is_loose) {
        const int rc = refresh_bound(c, s, nullptr);
        if (rc != SPKV_OK) return rc;
    }
    tighten_bound(c, s);
    const int rc = reserve_capacity(c, nullptr, s);
    if (rc != SPKV_OK) return rc;
    // the predictor's workgroups share the launch: leave them room in the resident round
    const int n_pred = spkv_predict_blocks(c->cfg.batch, d_hidden);
    c->split = choose_split(c, std::max(c->carve.n_pairs, c->one_round_items - n_pred),
                            c->carve.max_items);
    SpkvPredict pr = {};
    pr.x = static_cast<const uint16_t*>(hidden);
    pr.w1 = static_cast<const uint16_t*>(w1);
    pr.b1 = b1;
    pr.w2 = static_cast<const uint16_t*>(w2);
    pr.b2 = b2;
    pr.part = static_cast<float*>(workspace);
    pr.logits = util_logits;
    pr.d_model = d_model;
    pr.d_hidden = d_hidden;
    if (spkv_launch_decode_step_predict(c->view, static_cast<const uint16_t*>(k),
                                        static_cast<const uint16_t*>(v),
                                        static_cast<const uint16_t*>(q), static_cast<uint16_t*>(out),
                                        lse, sm_scale, c->split, pr, s) != hipSuccess)
        return SPKV_E_HIP;
    commit_lengths(c, nullptr);
    return SPKV_OK;
}

int spkv_decode_attention(spkv_cache_t* c, const void* q, void* out, float* lse, float sm_scale,
                          void* stream) {
    if (c == nullptr || q == nullptr || out == nullptr) return SPKV_E_INVAL;
    if (!aligned16(q) || !aligned16(out) || (lse != nullptr && !aligned16(lse))) return SPKV_E_INVAL;
    for (int b = 0; b < c->cfg.batch; ++b)
        if (c->T[b] == 0) return SPKV_E_STATE;
    if (!(sm_scale > 0.f)) sm_scale = 1.0f / std::sqrt((float)c->cfg.head_dim);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (c->bound_is_loose) {   // first decode after a bulk append: one read-back of the lengths
        const int rc = refresh_bound(c, s, nullptr);
        if (rc != SPKV_OK) return rc;
    }
    tighten_bound(c, s);
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    if (c->timing && c->n_timed < kMaxTimedLaunches) {
        if ((size_t)(2 * c->n_timed + 2) > c->events.size()) {
            hipEvent_t a, b2;
            if (hipEventCreate(&a) != hipSuccess) return SPKV_E_HIP;
            if (hipEventCreate(&b2) != hipSuccess) {
                (void)hipEventDestroy(a);
                return SPKV_E_HIP;
            }
            c->events.push_back(a);
            c->events.push_back(b2);
        }
        ev0 = c->events[2 * c->n_timed];
        ev1 = c->events[2 * c->n_timed + 1];
        c->n_timed += 1;
    }
    c->split = choose_split(c);
    if (spkv_launch_decode(c->view, static_cast<const uint16_t*>(q), static_cast<uint16_t*>(out),
                           lse, sm_scale, c->split, c->split_only, one_launch(c, s), ev0, ev1, s) != hipSuccess)
        return SPKV_E_HIP;
    return SPKV_OK;
}

int spkv_decode_attention_static(spkv_cache_t* c, const void* q, void* out, float* lse,
                                 float sm_scale, void* stream) {
    if (c == nullptr || q == nullptr || out == nullptr) return SPKV_E_INVAL;
    if (!aligned16(q) || !aligned16(out) || (lse != nullptr && !aligned16(lse))) return SPKV_E_INVAL;
    // partial slots the scratch holds for this shape: [cap][G][D] sums, then [cap][G][2]
    const int G = c->carve.G, D = c->cfg.head_dim;
    const int64_t cap = (int64_t)((kStaticScratchBytes - kAlign) / ((size_t)G * (D + 2) * sizeof(float)));
    if (cap < 2 * (int64_t)c->carve.n_pairs) return SPKV_E_CAPACITY;
    for (int b = 0; b < c->cfg.batch; ++b)
        if (c->T[b] == 0) return SPKV_E_STATE;
    if (c->bound_is_loose) return SPKV_E_STATE;      // would have to wait for the device
    char* base = static_cast<char*>(static_scratch_of_current_device());
    if (base == nullptr) return SPKV_E_HIP;
    if (!(sm_scale > 0.f)) sm_scale = 1.0f / std::sqrt((float)D);
    SpkvView v = c->view;
    v.part_acc = reinterpret_cast<float*>(base);
    v.part_ml = reinterpret_cast<float*>(base + align_up((size_t)cap * G * D * sizeof(float)));
    v.max_items = (int32_t)std::min<int64_t>(cap, INT32_MAX);
    c->split = choose_split(c, c->one_round_items, cap);
    if ((int64_t)c->carve.n_pairs * c->split.slots > cap) return SPKV_E_CAPACITY;
    if (spkv_launch_decode(v, static_cast<const uint16_t*>(q), static_cast<uint16_t*>(out), lse,
                           sm_scale, c->split, false, false, nullptr, nullptr,
                           static_cast<hipStream_t>(stream)) != hipSuccess)
        return SPKV_E_HIP;
    return SPKV_OK;
}

namespace {
int chunk_call(spkv_cache_t* c, const void* k, const void* v, const float* util_logits,
               const void* q, const int32_t* cu_seqlens, void* out, float* lse, float sm_scale,
               void* stream, bool append);
int prefill_core(spkv_cache_t* c, const void* k, const void* v, const float* util_logits,
                 const void* q, const int32_t* cu_seqlens, int n_max, void* out, float* lse,
                 float sm_scale, uint16_t* stage, int32_t* prefix, int shp, float* part,
                 size_t part_bytes, bool exact_fit, hipStream_t s);
}

int spkv_decode_chunk(spkv_cache_t* c, const void* k, const void* v, const float* util_logits,
                      const void* q, const int32_t* cu_seqlens, void* out, float* lse,
                      float sm_scale, void* stream) {
    return chunk_call(c, k, v, util_logits, q, cu_seqlens, out, lse, sm_scale, stream, true);
}

int spkv_score_chunk(spkv_cache_t* c, const void* k, const void* v, const void* q,
                     const int32_t* cu_seqlens, void* out, float* lse, float sm_scale, void* stream) {
    return chunk_call(c, k, v, nullptr, q, cu_seqlens, out, lse, sm_scale, stream, false);
}

namespace {
int chunk_call(spkv_cache_t* c, const void* k, const void* v, const float* util_logits,
               const void* q, const int32_t* cu_seqlens, void* out, float* lse, float sm_scale,
               void* stream, bool append) {
    if (c == nullptr || cu_seqlens == nullptr) return SPKV_E_INVAL;
    const int B = c->cfg.batch, G = c->carve.G;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (cu_seqlens[0] != 0) return SPKV_E_INVAL;
    int n_max = 0;
    for (int b = 0; b < B; ++b) {
        const int64_t n = (int64_t)cu_seqlens[b + 1] - cu_seqlens[b];
        if (n < 0 || n > SPKV_MAX_CHUNK_TOKENS || n > c->cfg.window || n * G > 64) return SPKV_E_INVAL;
        n_max = std::max(n_max, (int)n);
    }
    if (n_max == 0) return SPKV_OK;
    if (k == nullptr || v == nullptr || (append && util_logits == nullptr) || q == nullptr ||
        out == nullptr)
        return SPKV_E_INVAL;
    if (!aligned16(k) || !aligned16(v) || (append && !aligned16(util_logits)) || !aligned16(q) ||
        !aligned16(out) || (lse != nullptr && !aligned16(lse)))
        return SPKV_E_INVAL;
    if (!(sm_scale > 0.f)) sm_scale = 1.0f / std::sqrt((float)c->cfg.head_dim);
    if (!c->bound_is_loose) tighten_bound(c, s);
    const int cols = n_max * G;
    const int groups = cols <= 16 ? 1 : (cols <= 32 ? 2 : 4);
    if (append && groups > 1) {
        // More than one group of 16 query columns: the prefill kernels (tiles shared by a
        // workgroup through LDS) are the faster way to the same result; their staging rows and
        // prefix counts live in the cache's arena, the split-K partials in its partial buffers.
        return prefill_core(c, k, v, util_logits, q, cu_seqlens, n_max, out, lse, sm_scale,
                            reinterpret_cast<uint16_t*>(c->arena + c->carve.chunk_stage),
                            reinterpret_cast<int32_t*>(c->arena + c->carve.chunk_prefix),
                            c->carve.chunk_shp, c->view.part_acc,
                            (size_t)c->carve.max_items * G * c->cfg.head_dim * sizeof(float), false, s);
    }
    if (c->bound_is_loose) {       // the split-K partition below wants the exact lengths
        const int rc = refresh_bound(c, s, nullptr);
        if (rc != SPKV_OK) return rc;
    }
    if (append) {
        const int rc = reserve_capacity(c, cu_seqlens, s);
        if (rc != SPKV_OK) return rc;
    }

    const int gi = groups == 1 ? 0 : (groups == 2 ? 1 : 2);
    if (c->chunk_round_items[gi] == 0) {
        const int resident = spkv_chunk_resident_items(c->cfg.head_dim, groups);
        c->chunk_round_items[gi] = resident > 0 ? resident - resident / 24 : 960;
    }
    // every slot holds groups * 16 columns of partials instead of G
    const int64_t slot_cap = (int64_t)c->carve.max_items * G / (groups * 16);
    // With two or four column groups a wave needs most of the register file and only one or
    // two fit a SIMD; one resident round of such items then reads too little at a time, and
    // about 1 800 items (two rounds of the widest kernel) measured 12-15 % faster.
    c->split = choose_split_mw(c, std::max(c->chunk_round_items[gi], groups > 1 ? c->one_round_items * 5 / 8 : 0),
                               slot_cap, 1);

    // every slot the launch may write must lie inside the partial buffers (they are sized
    // for this at create; checked again here because an overrun would be a wild device write)
    if ((int64_t)c->carve.n_pairs * c->split.slots * groups * 16 > (int64_t)c->carve.max_items * G)
        return SPKV_E_CAPACITY;

    SpkvCu cu;
    std::memcpy(cu.v, cu_seqlens, (size_t)(B + 1) * 4);
    const uint16_t* kk = static_cast<const uint16_t*>(k);
    const uint16_t* vv = static_cast<const uint16_t*>(v);
    if (spkv_launch_decode_chunk(c->view, kk, vv, static_cast<const uint16_t*>(q),
                                 static_cast<uint16_t*>(out), lse, sm_scale, c->split, cu, groups,
                                 s) != hipSuccess)
        return SPKV_E_HIP;
    if (!append) return SPKV_OK;
    const hipError_t e = (n_max == 1)
                             ? spkv_launch_append_step(c->view, kk, vv, util_logits, cu, s)
                             : spkv_launch_append_bulk(c->view, kk, vv, util_logits, cu, n_max, nullptr, s);
    if (e != hipSuccess) return SPKV_E_HIP;
    commit_lengths(c, cu_seqlens);
    if (n_max > SPKV_MAX_CHUNK_TOKENS) c->bound_is_loose = true;   // short chunks: see tighten_bound
    return SPKV_OK;
}
}  // namespace

namespace {
// Few spans (short chunks, small batch) leave most of the chip idle while each workgroup
// walks a whole list: cut every span's tiles into ranges so that the launch has about as
// many workgroups as the chip holds at once -- one eight-wave workgroup per compute unit,
// two of four or two waves (measured: more ranges than that only add partial results to
// write and merge; 16 sequences x 16 tokens at 32k context, 175 us per call with four
// times as many, 150 us with this).
constexpr int kPrefillResident8 = 256, kPrefillResident = 512;
int prefill_split_cap(int spans, int nw) {
    const int resident = nw == 8 ? kPrefillResident8 : kPrefillResident;
    if (spans <= 0) return 1;
    return std::max(1, std::min(32, (resident + spans / 2) / spans));
}
}  // namespace

size_t spkv_prefill_workspace_bytes(const spkv_cache_t* c, int32_t max_tokens_per_sequence,
                                    int64_t max_total_tokens) {
    if (c == nullptr || max_tokens_per_sequence <= 0 || max_total_tokens <= 0) return 0;
    const size_t prefix = align_up((size_t)max_total_tokens * c->cfg.n_kv_heads * 4);
    const size_t shp = ((size_t)c->cfg.window + max_tokens_per_sequence + kHalfTokens - 1) / kHalfTokens;
    const size_t half_bytes = (size_t)2 * kHalfTokens * c->cfg.head_dim * 2;
    // Split-K partials.  A call cuts its spans into ks = round(resident / spans) ranges, which
    // is above one only while spans <= 2/3 resident, so it never holds more than 4/3 resident
    // workgroups of nw * 32 columns: 4/3 * 65536 columns (256 x 8 x 32 = 512 x 4 x 32),
    // whatever the chunk length.  Caches with more (sequence, head) pairs than that never split.
    const size_t partial = c->carve.n_pairs <= kPrefillResident * 2 / 3
                               ? align_up(((size_t)65536 * 4 / 3 + 64) * (c->cfg.head_dim + 2) * 4)
                               : 0;
    return prefix + align_up((size_t)c->carve.n_pairs * shp * half_bytes) + partial;
}

namespace {
// Prefill attention + append of a call whose arguments have been checked: staging rows,
// prefix counts and split-K partials in the buffers given (part_bytes: what `part` holds; the
// number of key ranges per span is cut down to what fits).  exact_fit: fail instead.
int prefill_core(spkv_cache_t* c, const void* k, const void* v, const float* util_logits,
                 const void* q, const int32_t* cu_seqlens, int n_max, void* out, float* lse,
                 float sm_scale, uint16_t* stage, int32_t* prefix, int shp, float* part,
                 size_t part_bytes, bool exact_fit, hipStream_t s) {
    const int B = c->cfg.batch;
    const int rc = reserve_capacity(c, cu_seqlens, s);
    if (rc != SPKV_OK) return rc;
    SpkvCu cu;
    std::memcpy(cu.v, cu_seqlens, (size_t)(B + 1) * 4);
    // split-K over every span's tiles when the spans alone would not fill the chip; each
    // range keeps at least a few tiles (lengths from the host's upper bound)
    const int spans = spkv_prefill_spans(c->carve.n_pairs, c->carve.G, n_max);
    int64_t tiles = 0;
    for (int p = 0; p < c->carve.n_pairs; ++p) tiles = std::max<int64_t>(tiles, c->L_ub[p] / kHalfTokens);
    tiles += (c->cfg.window + 64) / kHalfTokens;
    const SpkvPrefillShape sh = spkv_prefill_shape(c->carve.G, n_max);
    int ks = (int)std::max<int64_t>(1, std::min<int64_t>(prefill_split_cap(spans, sh.nw), tiles / 4));
    // exactly what this call writes must fit
    while (spkv_prefill_partial_bytes(spans, ks, sh, c->cfg.head_dim) > part_bytes) {
        if (exact_fit) return SPKV_E_INVAL;
        ks -= 1;                    // ks = 1 writes no partials
    }
    if (spkv_launch_prefill(c->view, static_cast<const uint16_t*>(k), static_cast<const uint16_t*>(v),
                            util_logits, static_cast<const uint16_t*>(q), static_cast<uint16_t*>(out),
                            lse, sm_scale, cu, n_max, stage, prefix, shp, ks, part, s) != hipSuccess)
        return SPKV_E_HIP;
    commit_lengths(c, cu_seqlens);
    if (n_max > SPKV_MAX_CHUNK_TOKENS) c->bound_is_loose = true;   // short chunks: see tighten_bound
    return SPKV_OK;
}
}  // namespace

int spkv_prefill_attention(spkv_cache_t* c, const void* k, const void* v, const float* util_logits,
                           const void* q, const int32_t* cu_seqlens, void* out, float* lse,
                           float sm_scale, void* workspace, size_t workspace_bytes, void* stream) {
    if (c == nullptr || cu_seqlens == nullptr) return SPKV_E_INVAL;
    const int B = c->cfg.batch;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (cu_seqlens[0] != 0) return SPKV_E_INVAL;
    int n_max = 0;
    for (int b = 0; b < B; ++b) {
        const int64_t n = (int64_t)cu_seqlens[b + 1] - cu_seqlens[b];
        if (n < 0) return SPKV_E_INVAL;
        n_max = std::max<int64_t>(n_max, n);
    }
    if (n_max == 0) return SPKV_OK;
    bool one_each = true;
    for (int b = 0; b < B; ++b) one_each = one_each && cu_seqlens[b + 1] - cu_seqlens[b] == 1;
    if (one_each)       // a plain decode step
        return spkv_decode_step(c, k, v, util_logits, q, out, lse, sm_scale, stream);
    // The shortest chunks go to the multi-token step: with one group of 16 query columns its
    // one-wave items read the lists at the decode step's rate, and it needs fewer launches
    // (measured on 16 sequences of 32k tokens: 2 tokens 122 us against 140 us here, 4 tokens
    // 128 against 140, 8 tokens 144 against 141; on 4 sequences of 128k this call is ahead
    // from 2 tokens on, by 4 %).
    if (n_max <= SPKV_MAX_CHUNK_TOKENS && n_max <= c->cfg.window && n_max * c->carve.G <= 16)
        return spkv_decode_chunk(c, k, v, util_logits, q, cu_seqlens, out, lse, sm_scale, stream);
    if (k == nullptr || v == nullptr || util_logits == nullptr || q == nullptr || out == nullptr ||
        workspace == nullptr)
        return SPKV_E_INVAL;
    if (!aligned16(k) || !aligned16(v) || !aligned16(util_logits) || !aligned16(q) ||
        !aligned16(out) || (lse != nullptr && !aligned16(lse)) ||
        (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0)
        return SPKV_E_INVAL;
    if (cu_seqlens[B] <= 0) return SPKV_E_INVAL;
    if (!(sm_scale > 0.f)) sm_scale = 1.0f / std::sqrt((float)c->cfg.head_dim);
    char* ws = static_cast<char*>(workspace);
    const size_t prefix_bytes = align_up((size_t)cu_seqlens[B] * c->cfg.n_kv_heads * 4);
    const int shp = (c->cfg.window + n_max + kHalfTokens - 1) / kHalfTokens;
    const size_t stage_bytes =
        align_up((size_t)c->carve.n_pairs * shp * ((size_t)2 * kHalfTokens * c->cfg.head_dim * 2));
    if (prefix_bytes + stage_bytes > workspace_bytes) return SPKV_E_INVAL;
    return prefill_core(c, k, v, util_logits, q, cu_seqlens, n_max, out, lse, sm_scale,
                        reinterpret_cast<uint16_t*>(ws + prefix_bytes), reinterpret_cast<int32_t*>(ws), shp,
                        reinterpret_cast<float*>(ws + prefix_bytes + stage_bytes),
                        workspace_bytes - prefix_bytes - stage_bytes, true, s);
}

namespace {
// Workspace of spkv_soft_gated_attention: [zeros: n_pairs int32][bias][staging half-pages].
struct SoftCarve {
    size_t zeros, bias, stage, total;
    int shp, n_pairs;
};
bool soft_carve(int batch, int n_kv_heads, int head_dim, int window, int64_t n_max, SoftCarve* o) {
    if (batch < 1 || batch > SPKV_MAX_BATCH || n_kv_heads < 1 || (head_dim != 64 && head_dim != 128) ||
        window < 1 || window > (1 << 20) || n_max < 1 || n_max > (1 << 30) ||
        (int64_t)batch * n_kv_heads > 16384)
        return false;
    o->n_pairs = batch * n_kv_heads;
    o->shp = (int)((window + n_max + kHalfTokens - 1) / kHalfTokens);
    const size_t half_bytes = (size_t)2 * kHalfTokens * head_dim * 2;
    o->zeros = 0;
    o->bias = align_up((size_t)o->n_pairs * 4);
    o->stage = o->bias + align_up((size_t)o->n_pairs * o->shp * kHalfTokens * 4);
    o->total = o->stage + (size_t)o->n_pairs * o->shp * half_bytes;
    return true;
}
}  // namespace

size_t spkv_soft_gated_workspace_bytes(int32_t batch, int32_t n_kv_heads, int32_t head_dim,
                                       int32_t window, int32_t max_tokens_per_sequence) {
    SoftCarve k;
    return soft_carve(batch, n_kv_heads, head_dim, window, max_tokens_per_sequence, &k) ? k.total : 0;
}

int spkv_soft_gated_attention(const void* q, const void* k, const void* v, const float* util_logits,
                              const int32_t* cu_seqlens, int32_t batch, int32_t n_q_heads,
                              int32_t n_kv_heads, int32_t head_dim, int32_t window, void* out,
                              float* lse, float sm_scale, void* workspace, size_t workspace_bytes,
                              void* stream) {
    if (cu_seqlens == nullptr || batch < 1 || batch > SPKV_MAX_BATCH || n_kv_heads < 1 ||
        n_q_heads < 1 || n_q_heads % n_kv_heads != 0 || n_q_heads / n_kv_heads > 16)
        return SPKV_E_INVAL;
    if (cu_seqlens[0] != 0) return SPKV_E_INVAL;
    int64_t n_max = 0;
    for (int b = 0; b < batch; ++b) {
        const int64_t n = (int64_t)cu_seqlens[b + 1] - cu_seqlens[b];
        if (n < 0) return SPKV_E_INVAL;
        n_max = std::max(n_max, n);
    }
    if (n_max == 0) return SPKV_OK;
    SoftCarve sc;
    if (!soft_carve(batch, n_kv_heads, head_dim, window, n_max, &sc)) return SPKV_E_INVAL;
    if (q == nullptr || k == nullptr || v == nullptr || util_logits == nullptr || out == nullptr ||
        workspace == nullptr || workspace_bytes < sc.total)
        return SPKV_E_INVAL;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(util_logits) || !aligned16(out) ||
        (lse != nullptr && !aligned16(lse)) || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0)
        return SPKV_E_INVAL;
    if (!(sm_scale > 0.f)) sm_scale = 1.0f / std::sqrt((float)head_dim);
    hipStream_t s = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    if (spkv_launch_fill_zero(ws + sc.zeros, sc.bias, s) != hipSuccess) return SPKV_E_HIP;
    // A view that only carries the shape: no sequence holds a token (t_pair = kept_len = 0),
    // so the kernels take every key from the staging rows of this call.
    SpkvView vw{};
    vw.B = batch;
    vw.Hq = n_q_heads;
    vw.Hkv = n_kv_heads;
    vw.G = n_q_heads / n_kv_heads;
    vw.D = head_dim;
    vw.w = window;
    vw.n_pairs = sc.n_pairs;
    vw.n_ring_pages = (window + kPageTokens - 1) / kPageTokens;
    vw.pt_cap = 1;
    vw.n_pages = 1;
    vw.t_pair = reinterpret_cast<int32_t*>(ws + sc.zeros);
    vw.kept_len = vw.t_pair;
    vw.page_table = vw.t_pair;
    vw.pool = reinterpret_cast<uint16_t*>(ws + sc.stage);
    vw.ring = vw.pool;
    SpkvCu cu;
    std::memcpy(cu.v, cu_seqlens, (size_t)(batch + 1) * 4);
    if (spkv_launch_soft_gated(vw, static_cast<const uint16_t*>(k), static_cast<const uint16_t*>(v),
                               util_logits, static_cast<const uint16_t*>(q), static_cast<uint16_t*>(out),
                               lse, sm_scale, cu, (int)n_max, reinterpret_cast<uint16_t*>(ws + sc.stage),
                               reinterpret_cast<float*>(ws + sc.bias), sc.shp, s) != hipSuccess)
        return SPKV_E_HIP;
    return SPKV_OK;
}

namespace {
// Pool pages the host's bound would reach after `n` more single-token steps of every
// sequence with every pair that leaves a window kept.
int64_t pages_after_steps(const spkv_cache* c, int64_t n) {
    const int B = c->cfg.batch, Hkv = c->cfg.n_kv_heads, w = c->cfg.window;
    int64_t pages = 0;
    for (int b = 0; b < B; ++b) {
        const int64_t ev = std::max<int64_t>(0, (int64_t)c->T[b] + n - w) -
                           std::max<int64_t>(0, (int64_t)c->T[b] - w);
        for (int h = 0; h < Hkv; ++h) pages += pages_for((int64_t)c->L_ub[b * Hkv + h] + ev);
    }
    return pages;
}
}  // namespace

int spkv_cache_safe_steps(spkv_cache_t* c, void* stream, int64_t* n_steps) {
    if (c == nullptr || n_steps == nullptr) return SPKV_E_INVAL;
    const int rc = refresh_bound(c, static_cast<hipStream_t>(stream), nullptr);
    if (rc != SPKV_OK) return rc;
    int64_t hi = INT64_MAX;
    for (int b = 0; b < c->cfg.batch; ++b)
        hi = std::min<int64_t>(hi, (int64_t)c->cfg.max_context - c->T[b]);
    hi = std::max<int64_t>(hi, 0);
    int64_t lo = 0;                      // largest n known to fit
    if (pages_after_steps(c, 0) > c->carve.n_pages) hi = 0;
    while (lo < hi) {                    // pages_after_steps is non-decreasing in n
        const int64_t mid = lo + (hi - lo + 1) / 2;
        if (pages_after_steps(c, mid) <= c->carve.n_pages) lo = mid;
        else hi = mid - 1;
    }
    *n_steps = lo;
    return SPKV_OK;
}

int spkv_cache_advance(spkv_cache_t* c, int64_t n_steps) {
    if (c == nullptr || n_steps < 0) return SPKV_E_INVAL;
    if (n_steps == 0) return SPKV_OK;
    for (int b = 0; b < c->cfg.batch; ++b)
        if ((int64_t)c->T[b] + n_steps > c->cfg.max_context) return SPKV_E_CAPACITY;
    if (pages_after_steps(c, n_steps) > c->carve.n_pages) return SPKV_E_CAPACITY;
    const int B = c->cfg.batch, Hkv = c->cfg.n_kv_heads, w = c->cfg.window;
    for (int b = 0; b < B; ++b) {
        const int64_t ev = std::max<int64_t>(0, (int64_t)c->T[b] + n_steps - w) -
                           std::max<int64_t>(0, (int64_t)c->T[b] - w);
        c->T[b] += (int32_t)n_steps;
        for (int h = 0; h < Hkv; ++h) {
            int32_t& L = c->L_ub[b * Hkv + h];
            c->pages_ub += pages_for((int64_t)L + ev) - pages_for(L);
            L += (int32_t)ev;
        }
        c->slack += ev * Hkv;
        c->snap_ev[b] += (int32_t)ev;
    }
    return SPKV_OK;
}

int spkv_cache_stats(spkv_cache_t* c, spkv_stats_t* st, int32_t* kept_len, void* stream) {
    if (c == nullptr || st == nullptr) return SPKV_E_INVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int n_pairs = c->carve.n_pairs, Hkv = c->cfg.n_kv_heads, w = c->cfg.window;
    std::vector<int32_t> len(n_pairs), gate(n_pairs);
    int rc = refresh_bound(c, s, len.data());
    if (rc != SPKV_OK) return rc;
    int32_t pool_next = 0, free_top = 0, err = 0;
    if (hipMemcpy(gate.data(), c->view.gate_on, (size_t)n_pairs * 4, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(&pool_next, c->view.pool_next, 4, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(&free_top, c->view.free_top, 4, hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemcpy(&err, c->view.err_flag, 4, hipMemcpyDeviceToHost) != hipSuccess)
        return SPKV_E_HIP;
    std::memset(st, 0, sizeof(*st));
    for (int b = 0; b < c->cfg.batch; ++b) {
        st->total_tokens += c->T[b];
        st->evicted_tokens += (int64_t)std::max(0, c->T[b] - w) * Hkv;
        st->window_tokens += (int64_t)std::min(c->T[b], w) * Hkv;
    }
    for (int p = 0; p < n_pairs; ++p) {
        st->kept_tokens += len[p];
        st->gate_on_tokens += gate[p];
    }
    st->density_evicted = st->evicted_tokens ? (double)st->kept_tokens / (double)st->evicted_tokens : 0.0;
    st->density_all = st->total_tokens ? (double)st->gate_on_tokens / ((double)st->total_tokens * Hkv) : 0.0;
    const int64_t row_bytes = (int64_t)2 * c->cfg.head_dim * 2;
    st->kept_kv_bytes = (st->kept_tokens + st->window_tokens) * row_bytes;
    st->dense_kv_bytes = st->total_tokens * Hkv * row_bytes;
    st->pool_pages_used = (int64_t)pool_next - free_top;
    st->pool_pages_total = c->carve.n_pages;
    st->arena_bytes = (int64_t)c->arena_bytes;
    st->device_error = err;
    const SpkvSplit sp = choose_split(c);   // the partition the next decode call would use
    int64_t n_items = 0;
    for (int p = 0; p < n_pairs; ++p) {
        const int Tw = std::min(c->T[p / Hkv], w);
        const int64_t hp = (len[p] + kHalfTokens - 1) / kHalfTokens + (Tw + kHalfTokens - 1) / kHalfTokens;
        const int64_t per = (int64_t)sp.hp_per_item * sp.mw;
        n_items += std::min<int64_t>(std::min<int64_t>((hp + per - 1) / per, sp.slots) * sp.mw, hp);
    }
    st->n_work_items = (int32_t)n_items;
    {   // the same count under the partition the most recent decode call actually used
        const SpkvSplit lp = c->split;
        int64_t n_last = 0;
        for (int p = 0; p < n_pairs; ++p) {
            const int Tw = std::min(c->T[p / Hkv], w);
            const int64_t hp = (len[p] + kHalfTokens - 1) / kHalfTokens + (Tw + kHalfTokens - 1) / kHalfTokens;
            const int64_t per = (int64_t)lp.hp_per_item * lp.mw;
            n_last += std::min<int64_t>(std::min<int64_t>((hp + per - 1) / per, lp.slots) * lp.mw, hp);
        }
        st->n_work_items_last_call = (int32_t)n_last;
    }
    if (kept_len != nullptr) std::memcpy(kept_len, len.data(), (size_t)n_pairs * 4);
    return err ? SPKV_E_DEVICE : SPKV_OK;
}

int spkv_cache_release_sequence(spkv_cache_t* c, int32_t b, void* stream) {
    if (c == nullptr || b < 0 || b >= c->cfg.batch) return SPKV_E_INVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // Exact lengths first (synchronises): the host's page bound must drop by exactly what
    // the sequence gives back.
    const int rc = refresh_bound(c, s, nullptr);
    if (rc != SPKV_OK) return rc;
    if (spkv_launch_release_sequence(c->view, b, s) != hipSuccess) return SPKV_E_HIP;
    const int Hkv = c->cfg.n_kv_heads;
    for (int h = 0; h < Hkv; ++h) {
        int32_t& L = c->L_ub[b * Hkv + h];
        c->pages_ub -= pages_for(L);
        L = 0;
    }
    c->T[b] = 0;
    return SPKV_OK;
}

int spkv_cache_kept_positions(spkv_cache_t* c, int32_t b, int32_t h, int32_t* pos, int32_t cap,
                              int32_t* n, void* stream) {
    if (c == nullptr || n == nullptr || b < 0 || b >= c->cfg.batch || h < 0 ||
        h >= c->cfg.n_kv_heads || cap < 0)
        return SPKV_E_INVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int pair = b * c->cfg.n_kv_heads + h;
    if (spkv_launch_gather_positions(c->view, pair, s) != hipSuccess) return SPKV_E_HIP;
    if (hipStreamSynchronize(s) != hipSuccess) return SPKV_E_HIP;
    int32_t L = 0;
    if (hipMemcpy(&L, c->view.kept_len + pair, 4, hipMemcpyDeviceToHost) != hipSuccess) return SPKV_E_HIP;
    *n = L;
    if (L > cap || (L > 0 && pos == nullptr)) return SPKV_E_INVAL;
    if (L > 0 &&
        hipMemcpy(pos, c->view.pos_scratch, (size_t)L * 4, hipMemcpyDeviceToHost) != hipSuccess)
        return SPKV_E_HIP;
    return SPKV_OK;
}

int spkv_cache_threshold_logit(const spkv_cache_t* c, float* theta) {
    if (c == nullptr || theta == nullptr) return SPKV_E_INVAL;
    *theta = c->view.theta;
    return SPKV_OK;
}

int spkv_cache_set_tau(spkv_cache_t* c, float tau) {
    if (c == nullptr || tau != tau) return SPKV_E_INVAL;
    c->cfg.tau = tau;
    c->view.theta = logit_threshold(tau);
    return SPKV_OK;
}

int spkv_cache_prune(spkv_cache_t* c, void* stream) {
    if (c == nullptr) return SPKV_E_INVAL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (spkv_launch_prune(c->view, s) != hipSuccess) return SPKV_E_HIP;
    return refresh_bound(c, s, nullptr);      // exact lengths and page count again (synchronises)
}

int spkv_cache_set_option(spkv_cache_t* c, int32_t option, int64_t value) {
    if (c == nullptr) return SPKV_E_INVAL;
    switch (option) {
        case SPKV_OPT_ITEM_TARGET:
            if (value < 0 || value > kMaxItemTarget) return SPKV_E_INVAL;
            c->item_target = (int)value;
            return SPKV_OK;
        case SPKV_OPT_SPLIT_ONLY:
            c->split_only = value != 0;
            return SPKV_OK;
        case SPKV_OPT_MERGE_WAVES:
            if (value != 0 && value != 1 && value != 2 && value != 4) return SPKV_E_INVAL;
            c->merge_waves = (int)value;
            return SPKV_OK;
        case SPKV_OPT_STEP_LAUNCHES:
            if (value != 0 && value != 1 && value != 2) return SPKV_E_INVAL;
            c->step_launches = (int)value;
            return SPKV_OK;
        case SPKV_OPT_SINK_TOKENS:
            if (value < 0 || value > c->cfg.max_context) return SPKV_E_INVAL;
            for (int32_t t : c->T)
                if (t != 0) return SPKV_E_STATE;
            c->n_sink = (int)value;
            c->view.n_sink = (int)value;
            return SPKV_OK;
        case SPKV_OPT_KERNEL_TIMING:
            c->timing = value != 0;
            c->n_timed = 0;
            return SPKV_OK;
        default:
            return SPKV_E_INVAL;
    }
}

int spkv_cache_read_kernel_timing(spkv_cache_t* c, float* ms, int32_t cap, int32_t* n) {
    if (c == nullptr || n == nullptr || cap < 0 || (cap > 0 && ms == nullptr)) return SPKV_E_INVAL;
    const int count = std::min<int>(c->n_timed, cap);
    for (int i = 0; i < count; ++i) {
        if (hipEventSynchronize(c->events[2 * i + 1]) != hipSuccess) return SPKV_E_HIP;
        if (hipEventElapsedTime(&ms[i], c->events[2 * i], c->events[2 * i + 1]) != hipSuccess)
            return SPKV_E_HIP;
    }
    *n = count;
    c->n_timed = 0;
    return SPKV_OK;
}

int64_t spkv_debug_layout_offset(int32_t head_dim, int32_t is_v, int32_t kidx, int32_t d) {
    if ((head_dim != 64 && head_dim != 128) || kidx < 0 || kidx >= kPageTokens || d < 0 ||
        d >= head_dim)
        return -1;
    return is_v ? spkv_v_off(head_dim, kidx, d) : spkv_k_off(head_dim, kidx, d);
}

int spkv_utility_logits(const void* hidden, const void* w1, const float* b1, const void* w2,
                        const float* b2, float* logits, float* workspace, int32_t n_tokens,
                        int32_t d_model, int32_t d_hidden, int32_t n_kv_heads, void* stream) {
    if (hidden == nullptr || w1 == nullptr || w2 == nullptr || logits == nullptr ||
        workspace == nullptr)
        return SPKV_E_INVAL;
    if (n_tokens < 0 || n_tokens > (1 << 24) || d_model < 128 || d_model % 128 != 0 ||
        d_hidden < 16 || d_hidden % 16 != 0 || d_hidden > (1 << 16) || n_kv_heads < 1 ||
        n_kv_heads > 1024)
        return SPKV_E_INVAL;
    if (!aligned16(hidden) || !aligned16(w1) || !aligned16(w2) || !aligned16(logits) ||
        !aligned16(workspace))
        return SPKV_E_INVAL;
    if (n_tokens == 0) return SPKV_OK;
    return spkv_launch_predictor(static_cast<const uint16_t*>(hidden),
                                 static_cast<const uint16_t*>(w1), b1,
                                 static_cast<const uint16_t*>(w2), b2, logits, workspace, n_tokens,
                                 d_model, d_hidden, n_kv_heads,
                                 static_cast<hipStream_t>(stream)) == hipSuccess
               ? SPKV_OK
               : SPKV_E_HIP;
}

int spkv_debug_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (dst == nullptr || src == nullptr || (bytes & 15u) != 0 || !aligned16(dst) || !aligned16(src))
        return SPKV_E_INVAL;
    return spkv_launch_copy(dst, src, bytes, static_cast<hipStream_t>(stream)) == hipSuccess
               ? SPKV_OK
               : SPKV_E_HIP;
}

int spkv_debug_read(const void* src, size_t region_bytes, int32_t run_bytes, int64_t first_run,
                    int64_t n_runs, int64_t stride, int32_t n_workgroups, void* sink, void* stream) {
    if (src == nullptr || sink == nullptr || !aligned16(src) || !aligned16(sink)) return SPKV_E_INVAL;
    if (run_bytes < 16384 || run_bytes % 16384 != 0) return SPKV_E_INVAL;
    const int64_t total_runs = (int64_t)(region_bytes / (size_t)run_bytes);
    if (total_runs < 1 || n_runs < 1 || n_runs > total_runs || first_run < 0 || stride < 1 ||
        stride > ((int64_t)1 << 31) || first_run > ((int64_t)1 << 31) || total_runs > ((int64_t)1 << 31))
        return SPKV_E_INVAL;               // (first_run + i) * stride stays below 2^64
    if (n_workgroups < 1 || n_workgroups > (1 << 20)) return SPKV_E_INVAL;
    return spkv_launch_read(src, total_runs, run_bytes / 16384, first_run, n_runs, stride, n_workgroups,
                            sink, static_cast<hipStream_t>(stream)) == hipSuccess
               ? SPKV_OK
               : SPKV_E_HIP;
}

const char* spkv_strerror(int code) {
    switch (code) {
        case SPKV_OK: return "ok";
        case SPKV_E_INVAL: return "invalid argument";
        case SPKV_E_STATE: return "decode on a sequence that holds no token";
        case SPKV_E_CAPACITY: return "cache capacity (pool pages, page table or max_context) exceeded";
        case SPKV_E_HIP: return "HIP runtime error";
        case SPKV_E_NOMEM: return "host allocation failed";
        case SPKV_E_DEVICE: return "kernel flagged an inconsistent cache state";
        default: return "unknown error";
    }
}

}  // extern "C"
