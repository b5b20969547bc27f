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

