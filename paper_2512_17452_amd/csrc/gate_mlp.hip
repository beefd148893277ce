// Write-Gate MLP (Sec. 3.2, feature equation and gate equation), per token t and kv head h:
//     x = [ RMSNorm(k[t][h]) ; RMSNorm(k_rope[t][h]) ]
//     g = sigmoid( W2[h] . GELU( W1[h] x + b1[h] ) + b2[h] )
// with the exact GELU and an RMSNorm without learnable scale (the paper fixes neither).
//
// The first layer is a dense contraction (tokens x 2d x width per head) and runs on the
// matrix cores, transposed: H^T = W1 X^T with v_mfma_f32_32x32x16_bf16, rows = 32 hidden
// units of a chunk of W1 staged in LDS, columns = the 32 tokens of a wave, whose
// normalised features stay in registers as the second operand for the whole kernel.  A
// lane then owns one token column, so bias, GELU, the product with W2 and the sum over
// hidden units are per-lane work and the hidden layer never leaves the registers.
// The normalised features are rounded to bf16 (they are a matrix-core operand), which is
// what a bf16 model does with its RMSNorm output as well.
#include "wgkv_dev.h"

namespace wgkv {

typedef __attribute__((ext_vector_type(8))) __bf16 gm_bf16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 gm_bf16x2_t;
typedef __attribute__((ext_vector_type(16))) float gm_f32x16_t;

constexpr int kGmUnits = 32;   // hidden units per chunk of W1
constexpr int kGmTokens = 32;  // tokens per wave

// Exact GELU z * Phi(z) with erf from the formula of Abramowitz & Stegun 7.1.26,
// erf(x) = 1 - (a1 t + ... + a5 t^5) exp(-x^2), t = 1 / (1 + p x), x >= 0, whose absolute error is
// below 1.5e-7 (a fifth of the library routine's instruction count; the GELU is what bounds the
// kernel).  With q = 1 - erf(|z| / sqrt 2): Phi(z) = 1 - q/2 for z >= 0 and q/2 for z < 0, so no
// difference of nearly equal numbers is formed on the negative side.
__device__ __forceinline__ float gm_gelu(float z) {
    const float x = fabsf(z) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
    float p = fmaf(1.061405429f, t, -1.453152027f);
    p = fmaf(p, t, 1.421413741f);
    p = fmaf(p, t, -0.284496736f);
    p = fmaf(p, t, 0.254829592f);
    const float q = p * t * __builtin_amdgcn_exp2f(x * x * -1.4426950408889634f);
    return 0.5f * z * (z >= 0.f ? 2.0f - q : q);
}

__device__ __forceinline__ float gm_bf16_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

__device__ __forceinline__ uint32_t gm_pack(float lo, float hi) {
    gm_bf16x2_t t = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, t);
}

template <int D>
__global__ __launch_bounds__(256) void gate_mlp_mfma_kernel(const char *k, const char *kr, const char *W1,
                                                            const float *b1, const char *W2, const float *b2,
                                                            float eps, float *g_out, long long T, int Hkv,
                                                            int width) {
    constexpr int KS = 2 * D / 16;             // contraction slices of 16 features
    constexpr int kRow = 2 * D * 2 + 16;       // bytes per W1 row in LDS (padded against bank conflicts)
    constexpr int kRowPieces = 2 * D * 2 / 16;                  // 16-byte pieces per row
    constexpr int kPieces = kGmUnits * kRowPieces / 256;        // pieces of a chunk per thread
    static_assert(kPieces == 2 || kPieces == 4, "");
    __shared__ __attribute__((aligned(16))) char s_w1[2][kGmUnits * kRow];
    __shared__ __attribute__((aligned(16))) float s_b1[2][kGmUnits];
    __shared__ __attribute__((aligned(16))) float s_w2[2][kGmUnits];

    const int h = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 31, half = lane >> 5;
    const long long tok = ((long long)blockIdx.x * 4 + wave) * kGmTokens + n;
    const long long tok_c = tok < T ? tok : T - 1;  // rows past the end repeat the last token, unwritten

    // ---- features: this lane's token, the 8 features [16 ks + 8 half, +8) of every slice ----
    gm_bf16x8_t xv[KS];
#pragma unroll
    for (int part = 0; part < 2; part++) {
        const char *row = (part == 0 ? k : kr) + ((size_t)tok_c * Hkv + h) * (D * 2);
        uint4 raw[KS / 2];
        float ss = 0.f;
#pragma unroll
        for (int j = 0; j < KS / 2; j++) {
            raw[j] = *reinterpret_cast<const uint4 *>(row + (2 * j + half) * 16);
            const uint32_t w[4] = {raw[j].x, raw[j].y, raw[j].z, raw[j].w};
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const float a = gm_bf16_to_f32(w[e] & 0xffffu), b = gm_bf16_to_f32(w[e] >> 16);
                ss = fmaf(a, a, ss);
                ss = fmaf(b, b, ss);
            }
        }
        ss += __shfl_xor(ss, 32);  // the other half of the row
        const float r = 1.0f / sqrtf(ss / (float)D + eps);
#pragma unroll
        for (int j = 0; j < KS / 2; j++) {
            const uint32_t w[4] = {raw[j].x, raw[j].y, raw[j].z, raw[j].w};
            uint32_t o[4];
#pragma unroll
            for (int e = 0; e < 4; e++)
                o[e] = gm_pack(gm_bf16_to_f32(w[e] & 0xffffu) * r, gm_bf16_to_f32(w[e] >> 16) * r);
            xv[part * (KS / 2) + j] = __builtin_bit_cast(gm_bf16x8_t, make_uint4(o[0], o[1], o[2], o[3]));
        }
    }

    // ---- chunks of 32 hidden units: W1 rows, b1 and W2 through LDS, two buffers ----
    const int n_chunks = width / kGmUnits;
    uint4 w0, w1, w2, w3;  // this thread's pieces of the chunk on its way to LDS
    w2 = w3 = make_uint4(0u, 0u, 0u, 0u);
    float b1v = 0.f, w2v = 0.f;
    auto fetch = [&](int c) __attribute__((always_inline)) {
        const char *src = W1 + ((size_t)h * width + (size_t)c * kGmUnits) * (2 * D * 2);  // 32 consecutive rows
        w0 = *reinterpret_cast<const uint4 *>(src + ((size_t)0 * 256 + threadIdx.x) * 16);
        w1 = *reinterpret_cast<const uint4 *>(src + ((size_t)1 * 256 + threadIdx.x) * 16);
        if (kPieces > 2) {
            w2 = *reinterpret_cast<const uint4 *>(src + ((size_t)2 * 256 + threadIdx.x) * 16);
            w3 = *reinterpret_cast<const uint4 *>(src + ((size_t)3 * 256 + threadIdx.x) * 16);
        }
        if (threadIdx.x < kGmUnits) {
            const size_t u = (size_t)h * width + (size_t)c * kGmUnits + threadIdx.x;
            b1v = b1[u];
            w2v = gm_bf16_to_f32(*reinterpret_cast<const uint16_t *>(W2 + u * 2));
        }
    };
    auto put = [&](int buf, int p, const uint4 v) __attribute__((always_inline)) {
        const int piece = p * 256 + threadIdx.x;
        *reinterpret_cast<uint4 *>(&s_w1[buf][(piece / kRowPieces) * kRow + (piece % kRowPieces) * 16]) = v;
    };
    auto stage = [&](int buf) __attribute__((always_inline)) {
        put(buf, 0, w0);
        put(buf, 1, w1);
        if (kPieces > 2) {
            put(buf, 2, w2);
            put(buf, 3, w3);
        }
        if (threadIdx.x < kGmUnits) {
            s_b1[buf][threadIdx.x] = b1v;
            s_w2[buf][threadIdx.x] = w2v;
        }
    };
    fetch(0);
    stage(0);
    __syncthreads();
    float acc_logit = 0.f;
    for (int c = 0; c < n_chunks; c++) {
        const int buf = c & 1;
        if (c + 1 < n_chunks) fetch(c + 1);
        gm_f32x16_t hcol;
#pragma unroll
        for (int i = 0; i < 16; i++) hcol[i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {
            const gm_bf16x8_t wa =
                *reinterpret_cast<const gm_bf16x8_t *>(&s_w1[buf][n * kRow + (ks * 16 + half * 8) * 2]);
            hcol = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa, xv[ks], hcol, 0, 0, 0);
        }
        // register 4j+i of a lane holds hidden unit 8j + 4*half + i of the chunk, for its token
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const float4 bb = *reinterpret_cast<const float4 *>(&s_b1[buf][8 * j + 4 * half]);
            const float4 ww = *reinterpret_cast<const float4 *>(&s_w2[buf][8 * j + 4 * half]);
            acc_logit = fmaf(ww.x, gm_gelu(hcol[4 * j + 0] + bb.x), acc_logit);
            acc_logit = fmaf(ww.y, gm_gelu(hcol[4 * j + 1] + bb.y), acc_logit);
            acc_logit = fmaf(ww.z, gm_gelu(hcol[4 * j + 2] + bb.z), acc_logit);
            acc_logit = fmaf(ww.w, gm_gelu(hcol[4 * j + 3] + bb.w), acc_logit);
        }
        if (c + 1 < n_chunks) stage(buf ^ 1);
        __syncthreads();
    }
    acc_logit += __shfl_xor(acc_logit, 32);  // the other 16 units of every chunk
    if (half == 0 && tok < T) g_out[(size_t)tok * Hkv + h] = 1.0f / (1.0f + __expf(-(acc_logit + b2[h])));
}

// Any other shape or an fp32 model: one block per (token, kv head), one hidden unit per
// thread and turn, fp32 arithmetic.  With bf16 inputs the features are rounded to bf16 like
// in the matrix-core kernel, so both compute the same function.
template <int DT>
__global__ __launch_bounds__(256) void gate_mlp_generic_kernel(const char *k, const char *kr, const char *W1,
                                                               const float *b1, const char *W2, const float *b2,
                                                               float eps, float *g_out, int Hkv, int d, int width) {
    extern __shared__ float s_x[];  // 2d features, then 8 partial sums
    float *s_red = s_x + 2 * d;
    const long long t = blockIdx.x;
    const int h = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    auto ld = [&](const char *p, size_t i) -> float {
        return DT == WGKV_F32 ? reinterpret_cast<const float *>(p)[i]
                              : gm_bf16_to_f32(reinterpret_cast<const uint16_t *>(p)[i]);
    };
    for (int part = 0; part < 2; part++) {
        const char *src = part == 0 ? k : kr;
        const size_t row = ((size_t)t * Hkv + h) * d;
        float ss = 0.f;
        for (int e = threadIdx.x; e < d; e += 256) {
            const float v = ld(src, row + e);
            ss = fmaf(v, v, ss);
        }
        ss = group_sum<64>(ss);
        __syncthreads();
        if (lane == 0) s_red[wave] = ss;
        __syncthreads();
        ss = s_red[0] + s_red[1] + s_red[2] + s_red[3];
        const float r = 1.0f / sqrtf(ss / (float)d + eps);
        for (int e = threadIdx.x; e < d; e += 256) {
            float xn = ld(src, row + e) * r;
            if (DT == WGKV_BF16) xn = (float)(__bf16)xn;
            s_x[part * d + e] = xn;
        }
    }
    __syncthreads();
    float acc = 0.f;
    for (int u = threadIdx.x; u < width; u += 256) {
        const size_t wrow = ((size_t)h * width + u) * 2 * d;
        float z = b1[(size_t)h * width + u];
        for (int e = 0; e < 2 * d; e++) z = fmaf(ld(W1, wrow + e), s_x[e], z);
        acc = fmaf(ld(W2, (size_t)h * width + u), gm_gelu(z), acc);
    }
    acc = group_sum<64>(acc);
    __syncthreads();
    if (lane == 0) s_red[4 + wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        const float logit = s_red[4] + s_red[5] + s_red[6] + s_red[7] + b2[h];
        g_out[(size_t)t * Hkv + h] = 1.0f / (1.0f + __expf(-logit));
    }
}

hipError_t launch_gate_mlp(int dtype, int64_t n_tokens, int n_kv_heads, int head_dim, int width,
                           const void *k, const void *k_rope, const void *w1, const float *b1,
                           const void *w2, const float *b2, float eps, float *g_out, hipStream_t st) {
    if (n_tokens == 0) return hipSuccess;
    const char *kp = (const char *)k, *krp = (const char *)k_rope, *w1p = (const char *)w1, *w2p = (const char *)w2;
    if (dtype == WGKV_BF16 && (head_dim == 128 || head_dim == 64) && width % kGmUnits == 0) {
        const dim3 grid((unsigned)((n_tokens + 4 * kGmTokens - 1) / (4 * kGmTokens)), n_kv_heads);
        if (head_dim == 128)
            hipLaunchKernelGGL(gate_mlp_mfma_kernel<128>, grid, dim3(256), 0, st, kp, krp, w1p, b1, w2p, b2, eps,
                               g_out, (long long)n_tokens, n_kv_heads, width);
        else
            hipLaunchKernelGGL(gate_mlp_mfma_kernel<64>, grid, dim3(256), 0, st, kp, krp, w1p, b1, w2p, b2, eps,
                               g_out, (long long)n_tokens, n_kv_heads, width);
        return hipGetLastError();
    }
    // grid.x carries the tokens: split very long inputs over several launches
    const size_t smem = (size_t)(2 * head_dim + 8) * sizeof(float);
    const int es = dtype == WGKV_F32 ? 4 : 2;
    for (int64_t t0 = 0; t0 < n_tokens; t0 += (1 << 30)) {
        const int64_t nt = n_tokens - t0 < (1 << 30) ? n_tokens - t0 : (1 << 30);
        const dim3 grid((unsigned)nt, n_kv_heads);
        const size_t off = (size_t)t0 * n_kv_heads * head_dim * es;
        if (dtype == WGKV_F32)
            hipLaunchKernelGGL(gate_mlp_generic_kernel<WGKV_F32>, grid, dim3(256), smem, st, kp + off, krp + off, w1p,
                               b1, w2p, b2, eps, g_out + (size_t)t0 * n_kv_heads, n_kv_heads, head_dim, width);
        else
            hipLaunchKernelGGL(gate_mlp_generic_kernel<WGKV_BF16>, grid, dim3(256), smem, st, kp + off, krp + off,
                               w1p, b1, w2p, b2, eps, g_out + (size_t)t0 * n_kv_heads, n_kv_heads, head_dim, width);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace wgkv
