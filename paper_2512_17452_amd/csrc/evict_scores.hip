// Importance scores for budgeted eviction (appendix "Eviction policy implementation"),
// per (sequence, kv head), over the N entries of the head's global cache and the queries
// of an observation window (n_obs positions x G query heads of the group):
//   (1) A = Softmax(Q_obs K^T * scale), one softmax per query row over the N entries,
//   (2) S_raw_j = sum_i max_g A[(i,g)][j],
//   (3) S = MaxPool(S_raw, pool_w), centred, clipped at the ends of the cache.
// A softmax row needs its maximum and its denominator before any weight is final, so the
// keys are swept twice:
//   stats pass  : block = (unit, 64 query rows), all keys   -> (max, denominator) per row
//   weight pass : block = (unit, 64 keys), all query rows   -> S_raw of its keys
//   pool pass   : S from S_raw
// Every sum runs in a fixed order, so the scores (and what gets evicted) repeat run to run.
#include "wgkv_dev.h"

namespace wgkv {

constexpr int kEsTile = 64;   // rows / keys per tile
constexpr int kEsDk = 32;     // slice of head_dim staged per step

struct EvictScoreArgs {
    int layer;
    int n_obs;
    int pool_w;
    float scale_log2e;
    const char *q;        // [n_seqs][n_obs][Hq][d]
    float *stats;         // workspace [n_units][n_obs * G][2]
    float *raw;           // [n_units][stride]
    float *out;           // [n_units][stride]
    long long stride;
};

template <int DT>
__device__ __forceinline__ float es_ld(const char *p, size_t i) {
    return DT == WGKV_F32 ? reinterpret_cast<const float *>(p)[i]
                          : __uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(p)[i] << 16);
}

// acc[i][k] = q_row(row0 + 4 ty + i) . key(key0 + tx + 16 k), unscaled.  Rows / keys past the end count as zero.
template <int DT>
__device__ __forceinline__ void es_tile(const View &pv, const EvictScoreArgs &a, int um, int b, int h, int row0,
                                        int key0, int n_rows, int N, float (&acc)[4][4],
                                        float (*sq)[kEsDk + 1], float (*sk)[kEsDk + 1]) {
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int k = 0; k < 4; k++) acc[i][k] = 0.f;
    for (int d0 = 0; d0 < pv.d; d0 += kEsDk) {
        __syncthreads();
        for (int e = threadIdx.x; e < kEsTile * kEsDk; e += 256) {
            const int r = e / kEsDk, c = e % kEsDk;
            float qv = 0.f, kv = 0.f;
            if (d0 + c < pv.d) {
                const int row = row0 + r, key = key0 + r;
                if (row < n_rows) {
                    const int i = row / pv.G, g = row % pv.G;
                    qv = es_ld<DT>(a.q, (((size_t)b * a.n_obs + i) * pv.Hq + (size_t)h * pv.G + g) * pv.d + d0 + c);
                }
                if (key < N) {
                    const char *pg = page_ptr(pv, pv.global_pt[(size_t)um * pv.maxgp + (key >> pv.logP)]) +
                                     (size_t)(key & (pv.P - 1)) * pv.row_bytes;
                    kv = es_ld<DT>(pg, d0 + c);
                }
            }
            sq[r][c] = qv;
            sk[r][c] = kv;
        }
        __syncthreads();
#pragma unroll 8
        for (int c = 0; c < kEsDk; c++) {
            float qa[4], kb[4];
#pragma unroll
            for (int i = 0; i < 4; i++) qa[i] = sq[4 * ty + i][c];
#pragma unroll
            for (int k = 0; k < 4; k++) kb[k] = sk[tx + 16 * k][c];
#pragma unroll
            for (int i = 0; i < 4; i++)
#pragma unroll
                for (int k = 0; k < 4; k++) acc[i][k] = fmaf(qa[i], kb[k], acc[i][k]);
        }
    }
}

// (max, denominator) of every softmax row, in the base-2 exponent domain (score * scale * log2 e)
template <int DT>
__global__ __launch_bounds__(256) void evict_stats_kernel(View pv, CallSeqs cs, EvictScoreArgs a) {
    __shared__ float sq[kEsTile][kEsDk + 1], sk[kEsTile][kEsDk + 1];
    const int u = blockIdx.y, b = u / pv.Hkv, h = u % pv.Hkv;
    const int um = unit_meta(pv, cs.sid[b], a.layer, h);
    const int N = pv.global_len[um], n_rows = a.n_obs * pv.G;
    const int row0 = blockIdx.x * kEsTile;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float m[4], l[4];
#pragma unroll
    for (int i = 0; i < 4; i++) { m[i] = -INFINITY; l[i] = 0.f; }
    for (int key0 = 0; key0 < N; key0 += kEsTile) {
        float acc[4][4];
        es_tile<DT>(pv, a, um, b, h, row0, key0, n_rows, N, acc, sq, sk);
#pragma unroll
        for (int i = 0; i < 4; i++) {
            float x[4], mt = -INFINITY;
#pragma unroll
            for (int k = 0; k < 4; k++) {
                x[k] = (key0 + tx + 16 * k < N) ? acc[i][k] * a.scale_log2e : -INFINITY;
                mt = fmaxf(mt, x[k]);
            }
            // the 16 lanes tx = 0..15 of a row sit in one aligned group of 16 lanes
            mt = fmaxf(mt, __shfl_xor(mt, 1));
            mt = fmaxf(mt, __shfl_xor(mt, 2));
            mt = fmaxf(mt, __shfl_xor(mt, 4));
            mt = fmaxf(mt, __shfl_xor(mt, 8));
            const float mn = fmaxf(m[i], mt);  // finite: every tile has at least one key
            float ps = 0.f;
#pragma unroll
            for (int k = 0; k < 4; k++) ps += exp2f(x[k] - mn);
            ps = group_sum<16>(ps);
            l[i] = l[i] * exp2f(m[i] - mn) + ps;
            m[i] = mn;
        }
    }
    if (tx == 0)
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int row = row0 + 4 * ty + i;
            if (row < n_rows) {
                a.stats[((size_t)u * n_rows + row) * 2 + 0] = m[i];
                a.stats[((size_t)u * n_rows + row) * 2 + 1] = l[i];
            }
        }
}

// S_raw of 64 keys: all query rows in tiles of 64, weights through LDS for the maximum over the
// group and the sum over the observation window
template <int DT>
__global__ __launch_bounds__(256) void evict_weights_kernel(View pv, CallSeqs cs, EvictScoreArgs a) {
    __shared__ float sq[kEsTile][kEsDk + 1], sk[kEsTile][kEsDk + 1];
    __shared__ float sp[kEsTile][kEsTile + 1];   // weights of a tile: [row][key]
    __shared__ float s_part[4][kEsTile];
    const int u = blockIdx.y, b = u / pv.Hkv, h = u % pv.Hkv;
    const int um = unit_meta(pv, cs.sid[b], a.layer, h);
    const int N = pv.global_len[um], n_rows = a.n_obs * pv.G;
    const int key0 = blockIdx.x * kEsTile;
    if (key0 >= N) return;  // block-uniform
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int kj = threadIdx.x & 63, part = threadIdx.x >> 6;  // role in the reduction: key, quarter of the rows
    float sum = 0.f;
    for (int row0 = 0; row0 < n_rows; row0 += kEsTile) {
        float acc[4][4];
        es_tile<DT>(pv, a, um, b, h, row0, key0, n_rows, N, acc, sq, sk);
        __syncthreads();  // the previous tile's reduction is done with sp
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const int row = row0 + 4 * ty + i;
            float mr = 0.f, inv = 0.f;
            if (row < n_rows) {
                mr = a.stats[((size_t)u * n_rows + row) * 2 + 0];
                inv = 1.0f / a.stats[((size_t)u * n_rows + row) * 2 + 1];
            }
#pragma unroll
            for (int k = 0; k < 4; k++)
                sp[4 * ty + i][tx + 16 * k] = (row < n_rows) ? exp2f(acc[i][k] * a.scale_log2e - mr) * inv : 0.f;
        }
        __syncthreads();
        // rows of a tile are (observation row, head of the group) with the heads adjacent
        for (int il = part; il < kEsTile / pv.G; il += 4) {
            float best = sp[il * pv.G][kj];
            for (int g = 1; g < pv.G; g++) best = fmaxf(best, sp[il * pv.G + g][kj]);
            sum += best;
        }
    }
    s_part[part][kj] = sum;
    __syncthreads();
    if (part == 0 && key0 + kj < N && key0 + kj < a.stride)  // never past the caller's row, whatever the device's length
        a.raw[(size_t)u * a.stride + key0 + kj] = ((s_part[0][kj] + s_part[1][kj]) + s_part[2][kj]) + s_part[3][kj];
}


// ---------------------------------------------------------------------------------------------
// Matrix-core versions of the two sweeps for the shape of the paper's models (bf16, head_dim 128,
// group of 4, n_obs a multiple of 8).  Scores are formed transposed, S^T = K Q^T with
// v_mfma_f32_32x32x16_bf16: rows = 32 keys of a tile staged in LDS, columns = 32 query rows of a
// wave, ordered (observation row, head) with the four heads of a row adjacent.  A lane then owns
// one query row: its maximum, denominator and normalisation are per-lane scalars, the maximum
// over the group is a maximum over the four lanes of a quad, and the sum over the window is a sum
// over quads and waves.
typedef __attribute__((ext_vector_type(8))) __bf16 es_bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float es_f32x16_t;
constexpr int kEmD = 128, kEmKT = 32, kEmRow = 272;  // bytes per key row in LDS: 256 + 16 of padding

// the eight operand slices of a lane's query row (column `col` of the unit), zeros past the end
__device__ __forceinline__ void em_load_q(const View &pv, const EvictScoreArgs &a, int b, int h, int col, int n_cols,
                                          int half, es_bf16x8_t (&qv)[8]) {
    const int cc = min(col, n_cols - 1), i = cc >> 2, g = cc & 3;
    const char *qp = a.q + (((size_t)b * a.n_obs + i) * pv.Hq + (size_t)h * 4 + g) * (kEmD * 2);
#pragma unroll
    for (int ks = 0; ks < 8; ks++) qv[ks] = *reinterpret_cast<const es_bf16x8_t *>(qp + (ks * 16 + half * 8) * 2);
}

__global__ __launch_bounds__(512) void evict_stats_mfma_kernel(View pv, CallSeqs cs, EvictScoreArgs a) {
    __shared__ __attribute__((aligned(16))) char s_k[2][kEmKT * kEmRow];
    const int u = blockIdx.y, b = u / pv.Hkv, h = u % pv.Hkv;
    const int um = unit_meta(pv, cs.sid[b], a.layer, h);
    const int N = pv.global_len[um], n_cols = a.n_obs * 4;
    if (N == 0) return;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 31, half = lane >> 5;
    const int col = (blockIdx.x * 8 + wave) * 32 + n;
    es_bf16x8_t qv[8];
    em_load_q(pv, a, b, h, col, n_cols, half, qv);
    // staging: thread -> (key of the tile, 16-byte chunk); page ids in a per-lane register
    const int ld_key = threadIdx.x >> 4, ld_c = threadIdx.x & 15;
    int pt_base = 0;
    int ptreg = (lane < pv.maxgp) ? pv.global_pt[(size_t)um * pv.maxgp + lane] : 0;
    uint4 kreg;
    auto fetch = [&](int t) __attribute__((always_inline)) {
        if (((t * kEmKT + kEmKT - 1) >> pv.logP) >= pt_base + 64) {
            pt_base = (t * kEmKT) >> pv.logP;
            ptreg = (pt_base + lane < pv.maxgp) ? pv.global_pt[(size_t)um * pv.maxgp + pt_base + lane] : 0;
        }
        const int idx = min(t * kEmKT + ld_key, N - 1);
        const int pg = __shfl(ptreg, (idx >> pv.logP) - pt_base);
        kreg = *reinterpret_cast<const uint4 *>(page_ptr(pv, pg) + (size_t)(idx & (pv.P - 1)) * (kEmD * 2) + ld_c * 16);
    };
    const int n_tiles = (N + kEmKT - 1) / kEmKT;
    fetch(0);
    *reinterpret_cast<uint4 *>(&s_k[0][ld_key * kEmRow + ld_c * 16]) = kreg;
    __syncthreads();
    float m = -INFINITY, l = 0.f;
    for (int t = 0; t < n_tiles; t++) {
        const int buf = t & 1;
        if (t + 1 < n_tiles) fetch(t + 1);
        es_f32x16_t s;
#pragma unroll
        for (int c = 0; c < 16; c++) s[c] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ks++) {
            const es_bf16x8_t ka = *reinterpret_cast<const es_bf16x8_t *>(&s_k[buf][n * kEmRow + (ks * 16 + half * 8) * 2]);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qv[ks], s, 0, 0, 0);
        }
        // register 4j+i of a lane holds key 8j + 4*half + i of the tile
        float x[16], mt = -INFINITY;
#pragma unroll
        for (int c = 0; c < 16; c++) x[c] = s[c] * a.scale_log2e;
        if (t == n_tiles - 1) {  // block-uniform: only the last tile can reach past the end of the cache
            const int k0 = t * kEmKT + 4 * half;
#pragma unroll
            for (int c = 0; c < 16; c++) x[c] = (k0 + 8 * (c >> 2) + (c & 3) < N) ? x[c] : -INFINITY;
        }
#pragma unroll
        for (int c = 0; c < 16; c++) mt = fmaxf(mt, x[c]);
        const float mn = fmaxf(m, mt);
        const float ms = mn == -INFINITY ? 0.f : mn;  // this half may hold no valid key of the last tile
        // the hardware exponential: one instruction, a relative error of about an ulp, 0 for -inf
        float ps = 0.f;
#pragma unroll
        for (int c = 0; c < 16; c++) ps += __builtin_amdgcn_exp2f(x[c] - ms);
        l = l * __builtin_amdgcn_exp2f(m - ms) + ps;
        m = mn;
        if (t + 1 < n_tiles) *reinterpret_cast<uint4 *>(&s_k[buf ^ 1][ld_key * kEmRow + ld_c * 16]) = kreg;
        __syncthreads();
    }
    // the two halves of the wave hold different keys of the same query row
    const float m2 = __shfl_xor(m, 32), l2 = __shfl_xor(l, 32);
    const float M = fmaxf(m, m2);  // finite: N > 0
    const float Lsum = l * exp2f(m - M) + l2 * exp2f(m2 - M);
    // per unit: first n_cols values M + log2(L), what the weight sweep subtracts in the exponent
    // (exp2(x - M) / L = exp2(x - (M + log2 L))), then the n_cols denominators
    if (half == 0 && col < n_cols) {
        a.stats[(size_t)u * n_cols * 2 + col] = M + log2f(Lsum);
        a.stats[(size_t)u * n_cols * 2 + n_cols + col] = Lsum;
    }
}

constexpr int kEmKeys = 128;  // keys per block of the weight sweep (4 tiles)

// The weight sweep forms S = Q K^T, the other way round: rows = 32 query rows of a turn, columns = 32 keys.  A lane
// then owns one key, and its 16 registers are four observation rows x the four heads of the group: the maximum
// over the group is a maximum over four registers of the lane (no cross-lane step per weight), the sum over
// the window a sum inside the lane, then over the two halves of the wave and over the waves, in a fixed order.
// A block holds 128 keys as matrix operands in registers for all its turns (4 products per query operand
// loaded); the four waves take the turns of 32 query rows in turn.  n_cols is a multiple of 32 (n_obs of 8).
__global__ __launch_bounds__(256, 2) void evict_weights_mfma_kernel(View pv, CallSeqs cs, EvictScoreArgs a) {
    __shared__ __attribute__((aligned(16))) char s_k[kEmKeys * kEmRow];
    __shared__ float s_acc[4][kEmKeys];
    const int u = blockIdx.y, b = u / pv.Hkv, h = u % pv.Hkv;
    const int um = unit_meta(pv, cs.sid[b], a.layer, h);
    const int N = pv.global_len[um], n_cols = a.n_obs * 4;
    const int key0 = blockIdx.x * kEmKeys;
    if (key0 >= N) return;  // block-uniform
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 31, half = lane >> 5;
    const float *off_u = a.stats + (size_t)u * n_cols * 2;
    // the first turn's query rows, on their way while the keys are staged
    es_bf16x8_t qv[8];
    em_load_q(pv, a, b, h, wave * 32 + n, n_cols, half, qv);
    // the block's keys into LDS, zero rows past the end of the cache: eight 16-byte pieces per thread, their page
    // ids requested together and then the pieces together (keys past the end read the last key: no branch around a load)
    {
        static_assert(kEmKeys * 16 == 8 * 256, "eight pieces per thread");
        int pg[8];
        uint4 v[8];
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const int key = min(key0 + ((int)threadIdx.x >> 4) + 16 * j, N - 1);
            pg[j] = pv.global_pt[(size_t)um * pv.maxgp + (key >> pv.logP)];
        }
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const int key = min(key0 + ((int)threadIdx.x >> 4) + 16 * j, N - 1);
            v[j] = *reinterpret_cast<const uint4 *>(page_ptr(pv, pg[j]) + (size_t)(key & (pv.P - 1)) * (kEmD * 2) +
                                                    (threadIdx.x & 15) * 16);
        }
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const int kl = ((int)threadIdx.x >> 4) + 16 * j;
            if (key0 + kl >= N) v[j] = make_uint4(0u, 0u, 0u, 0u);
            *reinterpret_cast<uint4 *>(&s_k[kl * kEmRow + (threadIdx.x & 15) * 16]) = v[j];
        }
    }
    __syncthreads();
    es_bf16x8_t kreg[4][8];
#pragma unroll
    for (int kt = 0; kt < 4; kt++)
#pragma unroll
        for (int ks = 0; ks < 8; ks++)
            kreg[kt][ks] = *reinterpret_cast<const es_bf16x8_t *>(&s_k[(kt * 32 + n) * kEmRow + (ks * 16 + half * 8) * 2]);
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    const int n_turns = n_cols >> 5;
    for (int qt = wave; qt < n_turns; qt += 4) {  // wave-uniform
        // the exponent offsets of the turn's rows arrive while its products run
        float4 off4[4];
#pragma unroll
        for (int j = 0; j < 4; j++) off4[j] = *reinterpret_cast<const float4 *>(off_u + qt * 32 + 8 * j + 4 * half);
        // register 4j+i of a product: query row 8j + 4*half + i of the turn = observation row 2j + half, head i
        auto weigh = [&](const es_f32x16_t &sc, float &sum) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const float p0 = __builtin_amdgcn_exp2f(fmaf(sc[4 * j], a.scale_log2e, -off4[j].x));
                const float p1 = __builtin_amdgcn_exp2f(fmaf(sc[4 * j + 1], a.scale_log2e, -off4[j].y));
                const float p2 = __builtin_amdgcn_exp2f(fmaf(sc[4 * j + 2], a.scale_log2e, -off4[j].z));
                const float p3 = __builtin_amdgcn_exp2f(fmaf(sc[4 * j + 3], a.scale_log2e, -off4[j].w));
                sum += fmaxf(fmaxf(p0, p1), fmaxf(p2, p3));
            }
        };
        es_f32x16_t s0, s1;
#pragma unroll
        for (int c = 0; c < 16; c++) { s0[c] = 0.f; s1[c] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < 8; ks++) s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qv[ks], kreg[0][ks], s0, 0, 0, 0);
#pragma unroll
        for (int ks = 0; ks < 8; ks++) s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qv[ks], kreg[1][ks], s1, 0, 0, 0);
        weigh(s0, acc[0]);
        es_f32x16_t s2, s3;
#pragma unroll
        for (int c = 0; c < 16; c++) { s2[c] = 0.f; s3[c] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < 8; ks++) s2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qv[ks], kreg[2][ks], s2, 0, 0, 0);
        weigh(s1, acc[1]);
#pragma unroll
        for (int ks = 0; ks < 8; ks++) s3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qv[ks], kreg[3][ks], s3, 0, 0, 0);
        // the turn's products are issued: the next turn's query rows are requested into the same registers
        // and arrive while the last weights of this turn are formed
        if (qt + 4 < n_turns) em_load_q(pv, a, b, h, (qt + 4) * 32 + n, n_cols, half, qv);
        weigh(s2, acc[2]);
        weigh(s3, acc[3]);
    }
    // the two halves of a wave hold different observation rows of the same key; then the waves
#pragma unroll
    for (int kt = 0; kt < 4; kt++) {
        const float v = acc[kt] + __shfl_xor(acc[kt], 32);
        if (half == 0) s_acc[wave][kt * 32 + n] = v;
    }
    __syncthreads();
    if (threadIdx.x < kEmKeys && key0 + threadIdx.x < N && key0 + threadIdx.x < a.stride)  // never past the caller's row
        a.raw[(size_t)u * a.stride + key0 + threadIdx.x] =
            ((s_acc[0][threadIdx.x] + s_acc[1][threadIdx.x]) + s_acc[2][threadIdx.x]) + s_acc[3][threadIdx.x];
}

__global__ __launch_bounds__(256) void evict_pool_kernel(View pv, CallSeqs cs, EvictScoreArgs a) {
    const int u = blockIdx.y, b = u / pv.Hkv, h = u % pv.Hkv;
    // the part of the cache that fits the caller's rows (all of it unless the host's bound is stale)
    const int N = (int)min((long long)pv.global_len[unit_meta(pv, cs.sid[b], a.layer, h)], (long long)a.stride);
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= N) return;
    const float *raw = a.raw + (size_t)u * a.stride;
    float best = raw[j];
    for (int jj = max(0, j - a.pool_w / 2); jj <= min(N - 1, j + a.pool_w / 2); jj++) best = fmaxf(best, raw[jj]);
    a.out[(size_t)u * a.stride + j] = best;
}

size_t evict_scores_ws_bytes(const View &pv, int n_units, int n_obs) {
    return (((size_t)n_units * n_obs * pv.G * 2 * sizeof(float)) + 255) / 256 * 256;
}

// max_len: upper bound of the units' lengths (sizes the grids; blocks past a unit's end return at once)
hipError_t launch_evict_scores(const View &pv, const CallSeqs &cs, int layer, const void *q_obs, int n_obs,
                               float scale, int pool_w, float *raw, float *out, int64_t stride, int64_t max_len,
                               void *ws, hipStream_t st) {
    const int n_units = cs.n * pv.Hkv;
    if (max_len <= 0) return hipSuccess;
    EvictScoreArgs a;
    a.layer = layer;
    a.n_obs = n_obs;
    a.pool_w = pool_w;
    a.scale_log2e = scale * 1.4426950408889634f;
    a.q = (const char *)q_obs;
    a.stats = (float *)ws;
    a.raw = raw;
    a.out = out;
    a.stride = stride;
    const int n_rows = n_obs * pv.G;
    const dim3 g_stats((n_rows + kEsTile - 1) / kEsTile, n_units);
    const dim3 g_keys((unsigned)((max_len + kEsTile - 1) / kEsTile), n_units);
    const dim3 g_pool((unsigned)((max_len + 255) / 256), n_units);
    if (pv.dtype == WGKV_BF16 && pv.d == kEmD && pv.G == 4 && n_obs % 8 == 0) {
        const dim3 g_stats_m((n_rows + 255) / 256, n_units);
        const dim3 g_keys_m((unsigned)((max_len + kEmKeys - 1) / kEmKeys), n_units);
        hipLaunchKernelGGL(evict_stats_mfma_kernel, g_stats_m, dim3(512), 0, st, pv, cs, a);
        hipLaunchKernelGGL(evict_weights_mfma_kernel, g_keys_m, dim3(256), 0, st, pv, cs, a);
    } else if (pv.dtype == WGKV_F32) {
        hipLaunchKernelGGL(evict_stats_kernel<WGKV_F32>, g_stats, dim3(256), 0, st, pv, cs, a);
        hipLaunchKernelGGL(evict_weights_kernel<WGKV_F32>, g_keys, dim3(256), 0, st, pv, cs, a);
    } else {
        hipLaunchKernelGGL(evict_stats_kernel<WGKV_BF16>, g_stats, dim3(256), 0, st, pv, cs, a);
        hipLaunchKernelGGL(evict_weights_kernel<WGKV_BF16>, g_keys, dim3(256), 0, st, pv, cs, a);
    }
    hipLaunchKernelGGL(evict_pool_kernel, g_pool, dim3(256), 0, st, pv, cs, a);
    return hipGetLastError();
}

}  // namespace wgkv
