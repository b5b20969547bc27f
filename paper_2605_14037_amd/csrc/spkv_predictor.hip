// Utility predictor of the SP-KV gate (Eq. 1) on gfx950.
#include "spkv_device.h"

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
    const f32x4 acc = predictor_contract(wrow, xrow, kq);   // kq is a multiple of 32 (d_model of 128)
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

// Many tokens (prompt processing): the whole predictor in one launch, register-tiled.  One
// workgroup per 64 tokens; wave wv owns hidden units 64 wv .. 64 wv + 63, so d_hidden / 64
// waves cover the hidden layer.  Each wave keeps a 64 x 64 (hidden x token) tile of fp32 sums
// in 16 MFMA accumulators and walks d_model in steps of 32: four 16-byte loads of W1 rows and
// four of token rows per lane feed 16 MFMAs (the operands of the next step are loaded before
// the MFMAs of the current one).  Bias and SiLU are applied in registers, the output layer is
// taken per wave over its 64 hidden units (16 products per lane, head and token group, then a
// sum over the four lane groups), and the waves' partial logits meet in LDS.
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void spkv_predictor_tiled(const uint16_t* __restrict__ x,
                                                             const uint16_t* __restrict__ w1,
                                                             const float* __restrict__ b1,
                                                             const uint16_t* __restrict__ w2,
                                                             const float* __restrict__ b2,
                                                             float* __restrict__ logits, int n_tokens,
                                                             int d_model, int d_hidden, int n_kv_heads) {
    extern __shared__ float s_logit[];                     // [waves][64 tokens][n_kv_heads]
    const int tid = threadIdx.x, lane = tid & 63, kc = lane >> 4, n = lane & 15;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6), n_waves = d_hidden / 64;
    const int t0 = blockIdx.x * 64, j0 = wv * 64;
    const uint16_t* wrow[4];
    const uint16_t* xrow[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        wrow[i] = w1 + (size_t)(j0 + i * 16 + n) * d_model + kc * 8;
        // (columns past the last token read the last token's row; their results are not stored)
        xrow[i] = x + (size_t)min(t0 + i * 16 + n, n_tokens - 1) * d_model + kc * 8;
    }
    f32x4 acc[4][4];
#pragma unroll
    for (int hs = 0; hs < 4; ++hs)
#pragma unroll
        for (int ts = 0; ts < 4; ++ts) acc[hs][ts] = (f32x4){0.f, 0.f, 0.f, 0.f};
    // KS steps of 32 along d_model per iteration; the operands of the next iteration are
    // loaded before the MFMAs of the current one (d_model is a multiple of 128)
    constexpr int KS = 2;
    uint4 a[KS][4], b[KS][4];
#pragma unroll
    for (int u = 0; u < KS; ++u)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[u][i] = *reinterpret_cast<const uint4*>(wrow[i] + u * 32);
            b[u][i] = *reinterpret_cast<const uint4*>(xrow[i] + u * 32);
        }
    for (int k = KS * 32; k <= d_model; k += KS * 32) {
        uint4 an[KS][4], bn[KS][4];
        const int kn = min(k, d_model - KS * 32);          // the last iteration reloads its own operands
#pragma unroll
        for (int u = 0; u < KS; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                an[u][i] = *reinterpret_cast<const uint4*>(wrow[i] + kn + u * 32);
                bn[u][i] = *reinterpret_cast<const uint4*>(xrow[i] + kn + u * 32);
            }
        __builtin_amdgcn_sched_barrier(0);     // keep the loads ahead of the MFMAs
#pragma unroll
        for (int u = 0; u < KS; ++u)
#pragma unroll
            for (int hs = 0; hs < 4; ++hs)
#pragma unroll
                for (int ts = 0; ts < 4; ++ts)
                    acc[hs][ts] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                        __builtin_bit_cast(bf16x8, a[u][hs]), __builtin_bit_cast(bf16x8, b[u][ts]),
                        acc[hs][ts], 0, 0, 0);
#pragma unroll
        for (int u = 0; u < KS; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[u][i] = an[u][i];
                b[u][i] = bn[u][i];
            }
    }
    // lane (kc, n) holds hidden units j0 + 16 hs + 4 kc + i of tokens t0 + 16 ts + n
#pragma unroll
    for (int hs = 0; hs < 4; ++hs)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float bias = b1 != nullptr ? b1[j0 + hs * 16 + 4 * kc + i] : 0.f;
#pragma unroll
            for (int ts = 0; ts < 4; ++ts) {
                const float h = acc[hs][ts][i] + bias;
                acc[hs][ts][i] = h / (1.f + __expf(-h));                           // SiLU
            }
        }
    for (int hd = 0; hd < n_kv_heads; ++hd) {
        float w[4][4];
#pragma unroll
        for (int hs = 0; hs < 4; ++hs)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const unsigned bits = w2[(size_t)hd * d_hidden + j0 + hs * 16 + 4 * kc + i];
                w[hs][i] = __builtin_bit_cast(float, bits << 16);
            }
#pragma unroll
        for (int ts = 0; ts < 4; ++ts) {
            float p = 0.f;
#pragma unroll
            for (int hs = 0; hs < 4; ++hs)
#pragma unroll
                for (int i = 0; i < 4; ++i) p += w[hs][i] * acc[hs][ts][i];
            p += __shfl_xor(p, 16);
            p += __shfl_xor(p, 32);
            if (kc == 0) s_logit[((size_t)wv * 64 + ts * 16 + n) * n_kv_heads + hd] = p;
        }
    }
    __syncthreads();
    for (int o = tid; o < 64 * n_kv_heads; o += 64 * n_waves) {
        const int tok = o / n_kv_heads, hd = o - tok * n_kv_heads;
        if (t0 + tok >= n_tokens) continue;
        float sum = b2 != nullptr ? b2[hd] : 0.f;
        for (int w8 = 0; w8 < n_waves; ++w8) sum += s_logit[((size_t)w8 * 64 + tok) * n_kv_heads + hd];
        logits[(size_t)(t0 + tok) * n_kv_heads + hd] = sum;
    }
}

// Many tokens, d_hidden <= 256: the same tiling with the operands staged through LDS.  The
// register-tiled kernel above fetches its MFMA operands straight from memory in 64-byte
// pieces, 16 cache lines per load instruction, and every wave fetches the token rows again;
// that, not the MFMAs, sets its speed.  Here a workgroup (one wave per 64 hidden units) copies
// a block of 64 elements of d_model -- 128 bytes of every W1 row and of every one of its 64
// token rows -- straight into LDS, eight lanes per row (whole cache lines, each fetched once
// per workgroup), one block ahead of the one it computes on.  Chunk c (16 bytes) of row r is
// stored at position c ^ (r & 7) of the row, so that the eight lanes of an operand read that
// share a bank phase hit eight different bank groups.
constexpr int kGemmTokens = 64;      // tokens per workgroup
constexpr int kGemmK = 64;           // elements of d_model per stage

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void spkv_predictor_gemm(
    const uint16_t* __restrict__ x, const uint16_t* __restrict__ w1, const float* __restrict__ b1,
    const uint16_t* __restrict__ w2, const float* __restrict__ b2, float* __restrict__ logits,
    int n_tokens, int d_model, int d_hidden, int n_kv_heads) {
    extern __shared__ __attribute__((aligned(16))) unsigned char s_raw[];
    const int tid = threadIdx.x, lane = tid & 63, kc = lane >> 4, n = lane & 15;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6), n_waves = d_hidden / 64;
    const int t0 = blockIdx.x * kGemmTokens;
    const int rows = d_hidden + kGemmTokens;               // rows of a stage: W1 rows, then token rows
    const unsigned stage_bytes = (unsigned)rows * 128;
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)s_raw;
    // this wave's copies: 8 rows (1 KB) per load, rows 8 i .. 8 i + 7 for i = wv, wv + n_waves, ...
    const int r_in = lane >> 3, c_in = (lane & 7) ^ r_in;  // row within the 8, chunk fetched (swizzle)
    auto copy_stage = [&](int k0, int buf) {
        for (int i = wv; i < rows / 8; i += n_waves) {
            const int r = i * 8 + r_in;
            const uint16_t* src = r < d_hidden
                                      ? w1 + (size_t)r * d_model
                                      : x + (size_t)min(t0 + r - d_hidden, n_tokens - 1) * d_model;
            load_row_to_lds(src + k0 + c_in * 8,
                            __builtin_amdgcn_readfirstlane(lds0 + (unsigned)buf * stage_bytes + (unsigned)i * 1024));
        }
    };
    f32x4 acc[4][4];
#pragma unroll
    for (int hs = 0; hs < 4; ++hs)
#pragma unroll
        for (int ts = 0; ts < 4; ++ts) acc[hs][ts] = (f32x4){0.f, 0.f, 0.f, 0.f};

    __builtin_amdgcn_s_waitcnt(0x0f70);          // nothing of ours is in flight yet: vmcnt(0)
    copy_stage(0, 0);
    wait_loads_but<0>();
    __syncthreads();
    const int n_stages = d_model / kGemmK;
    for (int st = 0; st < n_stages; ++st) {
        const int buf = st & 1;
        if (st + 1 < n_stages) copy_stage((st + 1) * kGemmK, buf ^ 1);
        const unsigned char* tile = s_raw + (size_t)buf * stage_bytes;
#pragma unroll
        for (int u = 0; u < 2; ++u) {            // two MFMA steps of 32 per stage
            bf16x8 a[4], b[4];
            const int c = 4 * u + kc;            // chunk of the row this lane feeds
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int ra = wv * 64 + i * 16 + n, rb = d_hidden + i * 16 + n;
                a[i] = *reinterpret_cast<const bf16x8*>(tile + ra * 128 + ((c ^ (ra & 7)) << 4));
                b[i] = *reinterpret_cast<const bf16x8*>(tile + rb * 128 + ((c ^ (rb & 7)) << 4));
            }
#pragma unroll
            for (int hs = 0; hs < 4; ++hs)
#pragma unroll
                for (int ts = 0; ts < 4; ++ts)
                    acc[hs][ts] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[hs], b[ts], acc[hs][ts], 0, 0, 0);
        }
        wait_loads_but<0>();
        __syncthreads();
    }
    // lane (kc, n) holds hidden units 64 wv + 16 hs + 4 kc + i of tokens t0 + 16 ts + n
    const int j0 = wv * 64;
#pragma unroll
    for (int hs = 0; hs < 4; ++hs)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float bias = b1 != nullptr ? b1[j0 + hs * 16 + 4 * kc + i] : 0.f;
#pragma unroll
            for (int ts = 0; ts < 4; ++ts) {
                const float h = acc[hs][ts][i] + bias;
                acc[hs][ts][i] = h / (1.f + __expf(-h));                           // SiLU
            }
        }
    float* s_logit = reinterpret_cast<float*>(s_raw);      // [waves][64 tokens][n_kv_heads]
    for (int hd = 0; hd < n_kv_heads; ++hd) {
        float w[4][4];
#pragma unroll
        for (int hs = 0; hs < 4; ++hs)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const unsigned bits = w2[(size_t)hd * d_hidden + j0 + hs * 16 + 4 * kc + i];
                w[hs][i] = __builtin_bit_cast(float, bits << 16);
            }
#pragma unroll
        for (int ts = 0; ts < 4; ++ts) {
            float p = 0.f;
#pragma unroll
            for (int hs = 0; hs < 4; ++hs)
#pragma unroll
                for (int i = 0; i < 4; ++i) p += w[hs][i] * acc[hs][ts][i];
            p += __shfl_xor(p, 16);
            p += __shfl_xor(p, 32);
            if (kc == 0) s_logit[((size_t)wv * 64 + ts * 16 + n) * n_kv_heads + hd] = p;
        }
    }
    __syncthreads();
    for (int o = tid; o < kGemmTokens * n_kv_heads; o += 64 * n_waves) {
        const int tok = o / n_kv_heads, hd = o - tok * n_kv_heads;
        if (t0 + tok >= n_tokens) continue;
        float sum = b2 != nullptr ? b2[hd] : 0.f;
        for (int w8 = 0; w8 < n_waves; ++w8) sum += s_logit[((size_t)w8 * 64 + tok) * n_kv_heads + hd];
        logits[(size_t)(t0 + tok) * n_kv_heads + hd] = sum;
    }
}

hipError_t spkv_launch_predictor(const uint16_t* x, const uint16_t* w1, const float* b1,
                                 const uint16_t* w2, const float* b2, float* logits, float* act,
                                 int n_tokens, int d_model, int d_hidden, int n_kv_heads,
                                 hipStream_t s) {
    // A workgroup of the LDS-staged kernel takes about 80 us for d_model = 4096 (64 stages, each
    // waiting for its copy), so it pays once there are enough tokens to fill the chip with
    // workgroups: 32 768 tokens 125 us, 4096 tokens 83 us (two-kernel path: 1.0 ms, 128 us).
    if (n_tokens >= 4096 && d_hidden % 64 == 0 && d_hidden <= 256 && d_model % kGemmK == 0 &&
        n_kv_heads <= 64) {
        const int n_waves = d_hidden / 64;
        const size_t lds = std::max((size_t)2 * (d_hidden + kGemmTokens) * 128,
                                    (size_t)n_waves * 64 * n_kv_heads * sizeof(float));
        // more than the 64 KB of dynamic LDS a kernel gets by default
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(spkv_predictor_gemm),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        spkv_predictor_gemm<<<dim3((n_tokens + kGemmTokens - 1) / kGemmTokens), dim3(64 * n_waves), lds, s>>>(
            x, w1, b1, w2, b2, logits, n_tokens, d_model, d_hidden, n_kv_heads);
        return hipGetLastError();
    }
    // Wider hidden layers (up to 512 units): the register-tiled kernel, about 120 us per
    // workgroup for d_model = 4096 (32 768 tokens: 242 us).
    if (n_tokens >= 4096 && d_hidden % 64 == 0 && d_hidden <= 512 && n_kv_heads <= 64) {
        const int n_waves = d_hidden / 64;
        const size_t lds = (size_t)n_waves * 64 * n_kv_heads * sizeof(float);
        spkv_predictor_tiled<<<dim3((n_tokens + 63) / 64), dim3(64 * n_waves), lds, s>>>(
            x, w1, b1, w2, b2, logits, n_tokens, d_model, d_hidden, n_kv_heads);
        return hipGetLastError();
    }
    spkv_predictor_hidden<<<dim3(d_hidden / 16, (n_tokens + 15) / 16), dim3(256), 0, s>>>(
        x, w1, b1, act, n_tokens, d_model, d_hidden);
    spkv_predictor_out<<<dim3(n_tokens * n_kv_heads), dim3(64), 0, s>>>(act, w2, b2, logits, d_hidden,
                                                                        n_kv_heads);
    return hipGetLastError();
}

