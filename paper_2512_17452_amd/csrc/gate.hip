// Linear write gate: g[t][h] = sigmoid(w[h] . x[t])  -- the gate equation of
// Sec. 3.2 with the hidden layer removed, as the chunked-prefill workload uses it.
// HBM-bound: every hidden row is read once with 16-byte loads; the weights of a
// 4 KiB-per-head slice sit in LDS and are shared by the rows of the block.
#include "wgkv_dev.h"

namespace wgkv {

typedef __attribute__((ext_vector_type(2))) __bf16 gate_bf16x2_t;

constexpr int kGateRows = 2;        // rows per wave
constexpr int kGateSlice = 256;     // 16-byte chunks per head per LDS slice

template <int DT>
__device__ __forceinline__ float dot16(const uint4 &a, const uint4 &b, float c) {
    const uint32_t x[4] = {a.x, a.y, a.z, a.w}, y[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int e = 0; e < 4; e++) {
        if (DT == WGKV_BF16)
            c = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(gate_bf16x2_t, x[e]),
                                                __builtin_bit_cast(gate_bf16x2_t, y[e]), c, false);
        else
            c = fmaf(__uint_as_float(x[e]), __uint_as_float(y[e]), c);
    }
    return c;
}

template <int DT, int HK>
__global__ __launch_bounds__(256) void gate_linear_kernel(const char *hidden, const char *w,
                                                          float *g_out, long long T, int Dh, int Hkv) {
    constexpr int ES = DT == WGKV_F32 ? 4 : 2;
    constexpr int EPL = 16 / ES;
    __shared__ uint4 s_w[HK * kGateSlice];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long row0 = ((long long)blockIdx.x * 4 + wave) * kGateRows;
    const int n_chunks = Dh / EPL;  // 16-byte chunks per row
    float acc[kGateRows][HK];
#pragma unroll
    for (int r = 0; r < kGateRows; r++)
#pragma unroll
        for (int h = 0; h < HK; h++) acc[r][h] = 0.f;
    for (int c0 = 0; c0 < n_chunks; c0 += kGateSlice) {
        __syncthreads();
        for (int i = threadIdx.x; i < HK * kGateSlice; i += 256) {
            const int h = i / kGateSlice, c = c0 + i % kGateSlice;
            uint4 z = {0u, 0u, 0u, 0u};
            if (h < Hkv && c < n_chunks) z = *reinterpret_cast<const uint4 *>(w + ((size_t)h * Dh) * ES + (size_t)c * 16);
            s_w[i] = z;
        }
        __syncthreads();
        for (int cc = lane; cc < kGateSlice && c0 + cc < n_chunks; cc += 64) {
            uint4 x[kGateRows];
#pragma unroll
            for (int r = 0; r < kGateRows; r++) {
                x[r] = make_uint4(0u, 0u, 0u, 0u);
                if (row0 + r < T) x[r] = *reinterpret_cast<const uint4 *>(hidden + ((size_t)(row0 + r) * Dh) * ES + (size_t)(c0 + cc) * 16);
            }
#pragma unroll
            for (int h = 0; h < HK; h++) {
                const uint4 wv = s_w[h * kGateSlice + cc];
#pragma unroll
                for (int r = 0; r < kGateRows; r++) acc[r][h] = dot16<DT>(x[r], wv, acc[r][h]);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < kGateRows; r++)
#pragma unroll
        for (int h = 0; h < HK; h++) {
            const float s = group_sum<64>(acc[r][h]);
            if (lane == 0 && h < Hkv && row0 + r < T) g_out[(size_t)(row0 + r) * Hkv + h] = 1.0f / (1.0f + __expf(-s));
        }
}

hipError_t launch_gate_linear(int dtype, int64_t n_tokens, int hidden_dim, int n_kv_heads,
                              const void *hidden, const void *w, float *g_out, hipStream_t st) {
    const int rows_per_block = 4 * kGateRows;
    const unsigned grid = (unsigned)((n_tokens + rows_per_block - 1) / rows_per_block);
#define WGKV_GATE(DTV, HKV)                                                                     \
    hipLaunchKernelGGL((gate_linear_kernel<DTV, HKV>), dim3(grid), dim3(256), 0, st,            \
                       (const char *)hidden, (const char *)w, g_out, (long long)n_tokens, hidden_dim, n_kv_heads)
    if (dtype == WGKV_BF16) {
        if (n_kv_heads <= 8) WGKV_GATE(WGKV_BF16, 8); else WGKV_GATE(WGKV_BF16, 16);
    } else {
        if (n_kv_heads <= 8) WGKV_GATE(WGKV_F32, 8); else WGKV_GATE(WGKV_F32, 16);
    }
#undef WGKV_GATE
    return hipGetLastError();
}

}  // namespace wgkv
