// Linear write gate: g[t][h] = sigmoid(w[h] . x[t])  -- the gate equation of
// Sec. 3.2 with the hidden layer removed, as the chunked-prefill workload uses it.
// HBM-bound: every hidden row is read once with 16-byte loads; the weights of all
// heads sit in LDS (64 KiB) and are shared by the 32 rows of the block.
#include "wgkv_dev.h"

namespace wgkv {

typedef __attribute__((ext_vector_type(2))) __bf16 gate_bf16x2_t;

constexpr int kGateRows = 4;         // rows per wave
constexpr int kGateWaves = 8;        // waves per block
constexpr int kGateLdsChunks = 4096; // 16-byte chunks of weights in LDS (64 KiB), all heads together
constexpr int kGateAhead = 3;        // row chunks requested this many iterations before they are used

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

// One block of 8 waves per compute unit; a wave takes four rows at a time, row
// quads are dealt round-robin over all waves of the launch.  The weights of all
// heads for a slice of the row (the whole row for 4096 bf16 features and 8 heads:
// staged once per block) sit in LDS; a lane owns the 16-byte chunks lane, lane+64,
// ... of its four rows.  The work of a wave is one sequence of steps (row quad,
// slice) x 64-chunk iterations, and the loads of the next three iterations are in
// flight while it multiplies, across the end of a step and of a row quad as well.
template <int DT, int HK>
__global__ __launch_bounds__(kGateWaves * 64) void gate_linear_kernel(const char *hidden, const char *w,
                                                                      float *g_out, long long T, int Dh,
                                                                      int Hkv) {
    constexpr int ES = DT == WGKV_F32 ? 4 : 2;
    constexpr int EPL = 16 / ES;
    constexpr int SLICE = kGateLdsChunks / HK;  // chunks per head per slice
    constexpr int ITERS = SLICE / 64;
    constexpr int NBUF = kGateAhead + 1;
    static_assert(ITERS % NBUF == 0 && kGateAhead <= ITERS, "the ring of row buffers must close over a step");
    __shared__ uint4 s_w[HK * SLICE];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n_chunks = Dh / EPL;  // 16-byte chunks per row
    const long long total_waves = (long long)gridDim.x * kGateWaves;
    const long long n_quads = (T + kGateRows - 1) / kGateRows;
    const int n_pass = (int)((n_quads + total_waves - 1) / total_waves);  // the same for every wave: barriers inside
    const int n_slices = (n_chunks + SLICE - 1) / SLICE;
    const long long n_steps = (long long)n_pass * n_slices;
    const long long quad0 = (long long)wave * gridDim.x + blockIdx.x;
    const size_t row_bytes = (size_t)Dh * ES;

    // Loads are unconditional (a lane with nothing to read reads the first chunk of the
    // matrix and drops it): a branch around a load makes the compiler wait for every
    // outstanding load at the next use, and nothing stays in flight.
    uint4 x[NBUF][kGateRows];
    auto fetch = [&](uint4(&dst)[kGateRows], long long step, int it) __attribute__((always_inline)) {
        const long long row0 = ((step / n_slices) * total_waves + quad0) * kGateRows;
        const int cw = (int)(step % n_slices) * SLICE + it * 64 + lane;
        const bool okc = step < n_steps && cw < n_chunks;
#pragma unroll
        for (int r = 0; r < kGateRows; r++) {
            const bool ok = okc && row0 + r < T;
            const uint4 v = load_once16(ok ? hidden + (size_t)(row0 + r) * row_bytes + (size_t)cw * 16 : hidden);
            dst[r] = make_uint4(ok ? v.x : 0u, ok ? v.y : 0u, ok ? v.z : 0u, ok ? v.w : 0u);
        }
    };
#pragma unroll
    for (int it = 0; it < kGateAhead; it++) fetch(x[it], 0, it);
    float acc[kGateRows][HK];
    for (long long step = 0; step < n_steps; step++) {
        const int sl = (int)(step % n_slices), c0 = sl * SLICE;
        const long long row0 = ((step / n_slices) * total_waves + quad0) * kGateRows;
        if (sl == 0) {
#pragma unroll
            for (int r = 0; r < kGateRows; r++)
#pragma unroll
                for (int h = 0; h < HK; h++) acc[r][h] = 0.f;
        }
        if (n_slices > 1 || step == 0) {
            __syncthreads();
            for (int i = threadIdx.x; i < HK * SLICE; i += kGateWaves * 64) {
                const int h = i / SLICE, c = c0 + i % SLICE;
                uint4 z = {0u, 0u, 0u, 0u};
                if (h < Hkv && c < n_chunks)
                    z = *reinterpret_cast<const uint4 *>(w + ((size_t)h * Dh) * ES + (size_t)c * 16);
                s_w[i] = z;
            }
            __syncthreads();
        }
#pragma unroll
        for (int it = 0; it < ITERS; it++) {
            if (it + kGateAhead < ITERS) fetch(x[(it + kGateAhead) % NBUF], step, it + kGateAhead);
            else fetch(x[(it + kGateAhead) % NBUF], step + 1, it + kGateAhead - ITERS);
            if (c0 + it * 64 < n_chunks) {  // wave-uniform: otherwise nothing of this iteration lies in the row
#pragma unroll
                for (int h = 0; h < HK; h++) {
                    const uint4 wv = s_w[h * SLICE + it * 64 + lane];
#pragma unroll
                    for (int r = 0; r < kGateRows; r++)
                        acc[r][h] = dot16<DT>(x[it % NBUF][r], wv, acc[r][h]);
                }
            }
        }
        if (sl == n_slices - 1) {
            // 64-lane sums of the NV = 4 x HK partial results, halving the number of values
            // with the number of lanes that share one: lane bit 5, then bit 4, then a sum over
            // the row of 16.  Row q of the wave ends with values j + NV/4 * (q & 1) + NV/2 * (q >> 1).
            constexpr int NV = kGateRows * HK;
            float u[NV / 2], y[NV / 4];
#pragma unroll
            for (int j = 0; j < NV / 2; j++) {
                const LanePair t = swap32(acc[j / HK][j % HK], acc[(j + NV / 2) / HK][(j + NV / 2) % HK]);
                u[j] = t.a + t.b;
            }
#pragma unroll
            for (int j = 0; j < NV / 4; j++) {
                const LanePair t = swap16(u[j], u[j + NV / 4]);
                y[j] = group_sum<16>(t.a + t.b);
            }
            const int q = lane >> 4;
            if ((lane & 15) == 0) {
#pragma unroll
                for (int j = 0; j < NV / 4; j++) {
                    const int idx = j + (NV / 4) * (q & 1) + (NV / 2) * (q >> 1), r = idx / HK, h = idx % HK;
                    if (h < Hkv && row0 + r < T) g_out[(size_t)(row0 + r) * Hkv + h] = 1.0f / (1.0f + __expf(-y[j]));
                }
            }
        }
    }
}

hipError_t launch_gate_linear(int dtype, int64_t n_tokens, int hidden_dim, int n_kv_heads,
                              const void *hidden, const void *w, float *g_out, hipStream_t st) {
    // compute units of each device, asked for once
    static int n_cu_of[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (n_cu_of[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
            return hipErrorInvalidDevice;
        n_cu_of[dev] = n;
    }
    const int n_cu = n_cu_of[dev];
    const int64_t rows_per_block = kGateWaves * kGateRows;
    const int64_t want = (n_tokens + rows_per_block - 1) / rows_per_block;
    const unsigned grid = (unsigned)(want < n_cu ? want : n_cu);
#define WGKV_GATE(DTV, HKV)                                                                              \
    hipLaunchKernelGGL((gate_linear_kernel<DTV, HKV>), dim3(grid), dim3(kGateWaves * 64), 0, st,         \
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
