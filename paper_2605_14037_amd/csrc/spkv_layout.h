// Page layout of the SP-KV cache on MI355X.
//
// A page holds SPKV_PAGE_TOKENS = 64 key/value pairs of one (sequence, KV head) and is
// split into two half-pages of 32 pairs.  A half-page is one contiguous block:
//   [ K block : 32 * D bf16 ][ V block : 32 * D bf16 ]          (8 KB + 8 KB at D = 128)
// Inside the blocks the elements are ordered so that every 1 KB a wavefront loads with
// one 128-bit load per lane (lane l reads bytes [16 l, 16 l + 16)) already IS an operand
// of v_mfma_f32_16x16x32_bf16, with no shuffle and no LDS staging:
//
//   Key order.  Key r (0..31) of a half-page is written r = 8 kc + 4 t + i with kc in 0..3,
//   t in 0..1, i in 0..3: K tile t holds, as its row m = 4 kc + i, the key 8 kc + 4 t + i.
//
//   K block = [t : 2][chunk : D/8][m : 16][8 bf16]
//     row m of tile t, head-dim elements d = 8 chunk .. 8 chunk + 7.  The 1 KB tile
//     (t, slab) = chunks 4 slab .. 4 slab + 3 gives lane (kc' = l / 16, m = l % 16) the
//     8 elements d = 32 slab + 8 kc' + e of row m: the A operand (rows = keys,
//     contraction over d) of  S[key][head] += K[key][d] * Q[head][d].
//
//   V block = [db : D/16][kc : 4][dr : 16][8 bf16],  element e = 4 t + i
//     holds V[key r = 8 kc + e][d = 16 db + dr]: eight CONSECUTIVE keys of one output
//     dimension.  The 1 KB tile db gives lane (kc, dr) those eight keys: the A operand
//     (rows = d, contraction over keys) of  O[d][head] += V[key][d] * P[key][head].  The key
//     order inside lane group kc is exactly the order in which the S accumulators of the
//     two K tiles leave lane (kc, head) -- rows 4 kc + i of tile t -- so the softmax
//     weights go from the first MFMA to the second without crossing lanes; and because a
//     16-byte V unit is eight consecutive keys, eight rows appended together fill whole
//     units (the bulk write path assembles them in LDS).
//
// The window ring uses the same page layout (slot s mod w -> page slot / 64, index
// slot % 64), so the decode kernel reads ring and long-term pages with the same code.
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define SPKV_HD __host__ __device__ __forceinline__
#else
#define SPKV_HD inline
#endif

constexpr int kPageTokens = 64;
constexpr int kHalfTokens = 32;

// bf16 elements in one page (K and V together) for head_dim D.
SPKV_HD int spkv_page_elems(int D) { return 2 * kPageTokens * D; }

// Element offset, from the start of the page, of K[kidx][d].
SPKV_HD int spkv_k_off(int D, int kidx, int d) {
    const int half = kidx >> 5, kc = (kidx >> 3) & 3, t = (kidx >> 2) & 1, i = kidx & 3;
    const int m = 4 * kc + i;
    return half * (2 * kHalfTokens * D) + (((t * (D >> 3) + (d >> 3)) << 4) + m) * 8 + (d & 7);
}

// Element offset, from the start of the page, of V[kidx][d].
SPKV_HD int spkv_v_off(int D, int kidx, int d) {
    const int half = kidx >> 5, kc = (kidx >> 3) & 3;
    return half * (2 * kHalfTokens * D) + kHalfTokens * D +
           (((((d >> 4) << 2) + kc) << 4) + (d & 15)) * 8 + (kidx & 7);
}
