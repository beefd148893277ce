// Training-time Write-Gated Attention (Sec. 3.2, "Write-Gated Attention" and "Log-space
// transformation for efficient training") on the gfx950 matrix cores: causal attention of a
// whole sequence with the additive bias
//     B_ij = log(m_ij + eps),   m_ij = max(1(i - j < W_local), g_j),
// forward with the row log-sum-exp, and the gradients with respect to q, k, v and g.
//
//   soft_attn_fwd_kernel       block = 64 query positions x the 4 query heads of a kv head,
//                              key tiles of 64 staged in LDS; S^T = K Q^T, O^T = V^T P^T
//   soft_attn_rowdot_kernel    D_i = dO_i . O_i per (position, query head)
//   soft_attn_bwd_dq_kernel    same blocking as the forward: S^T and dP^T = V dO^T per key tile,
//                              dS^T = P^T (dP^T - D), dQ^T += K^T dS^T
//   soft_attn_bwd_dkv_kernel   block = 128 keys of a kv head; its waves are (32 keys) x (role):
//                              role 0 recomputes S = Q K^T and P and accumulates dV^T += dO^T P;
//                              role 1, one tile behind, computes dP = dO V^T, takes P through LDS, forms dS and
//                              accumulates dK^T += Q^T dS and the sum that becomes dg
//
// All products are v_mfma_f32_32x32x16_bf16 with fp32 accumulation; every operand that is
// reused over the whole loop (the block's own rows) sits in registers, the streamed tiles
// go through LDS row-major once: products over d read rows of the staged tile, products that
// contract over positions read its columns with the transposing LDS load (ds_read_b64_tr_b16).
// A lane of an accumulator tile owns one column, so per-column quantities are plain scalars.
#include <algorithm>
#include <climits>

#include "wgkv_dev.h"

namespace wgkv {

typedef __attribute__((ext_vector_type(8))) __bf16 sa_bf16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 sa_bf16x2_t;
typedef __attribute__((ext_vector_type(16))) float sa_f32x16_t;

constexpr int kSaD = 128;       // head_dim
constexpr int kSaG = 4;         // query heads per kv head
constexpr int kSaQ = 64;        // query positions per block (forward, dQ)
constexpr int kSaT = 32;        // positions per streamed tile
constexpr int kSaKB = 128;      // keys per block (dK/dV)
constexpr int kSaRm = 272;      // bytes per row of a tile in LDS whose rows are read whole (256 + 16 pad)
constexpr int kSaCm = 320;      // bytes per row of a tile that is only read column-wise (256 + 64 pad): four
                                // rows and 64 bytes of each per half wave, spread over all banks

struct SoftSeqs {
    int32_t n;
    int32_t ntok[kMaxCallSeqs];
    int32_t base[kMaxCallSeqs];  // first packed row of the sequence
};

struct SoftArgs {
    int nx;                 // blocks per (sequence, kv head) of the launch
    int Hq, Hkv, W;
    float scale_log2e;      // scale * log2(e): scores are kept in base-2 units
    float scale;
    float eps;
    const char *q, *k, *v;  // bf16 [rows][heads][128]
    const float *g;         // [rows][Hkv]
    float *out;             // [rows][Hq][128]
    float *lse;             // [rows][Hq], natural logarithm
    // backward only
    const char *dout;       // bf16 [rows][Hq][128]
    float *rowdot;          // [rows][Hq]
    float *dq, *dk, *dv, *dg;
};

__device__ __forceinline__ uint32_t sa_pack(float lo, float hi) {
    sa_bf16x2_t t = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, t);
}

// The two bias values of a key in base-2 units: inside the window m = max(1, g), outside m = max(0, g).
__device__ __forceinline__ void sa_bias(float gj, float eps, float &b_in, float &b_out) {
    b_in = __log2f(fmaxf(1.0f, gj) + eps);
    b_out = __log2f(fmaxf(0.0f, gj) + eps);
}

// One 16-byte chunk of a row goes to the row-major tile.
__device__ __forceinline__ void sa_put_rm(char *tile, int row, int dc, uint4 x) {
    *reinterpret_cast<uint4 *>(tile + row * kSaRm + dc * 16) = x;
}
// A operand of a product over d: row qn of a row-major tile, d slice ks.
__device__ __forceinline__ sa_bf16x8_t sa_get_rm(const char *tile, int qn, int half, int ks) {
    return *reinterpret_cast<const sa_bf16x8_t *>(tile + qn * kSaRm + (ks * 16 + half * 8) * 2);
}
// A operand of a product that contracts over the rows of a row-major tile (rows are positions,
// columns d): the output row of this lane is d = db*32 + qn, its 8 contraction slots are tile rows
// r0 + 4*half + {0..3} and r0 + 8 + 4*half + {0..3}, which is where the accumulator layout of the
// first product leaves this lane's values.  ds_read_b64_tr_b16 transposes inside groups of 16
// lanes: lane i of a group receives element i%4 of the 8 bytes addressed by lanes i/4, 4 + i/4,
// 8 + i/4 and 12 + i/4.  So lane s of a group addresses (row s/4 of the four, columns 4*(s%4)..+3 of
// the group's 16) and ends up with the four rows at its own column.
typedef short sa_s16x4_t __attribute__((ext_vector_type(4)));
template <int STRIDE = kSaRm>
__device__ __forceinline__ sa_bf16x8_t sa_get_cols(const char *tile, int lane, int db, int r0) {
    const int half = lane >> 5;
    const char *p = tile + (r0 + 4 * half + ((lane & 15) >> 2)) * STRIDE +
                    (db * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
    typedef sa_s16x4_t __attribute__((address_space(3))) *lds_ptr_t;
    const sa_s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)p);
    const sa_s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 8 * STRIDE));
    const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
    const uint4 u4 = make_uint4(l2.x, l2.y, h2.x, h2.y);
    return __builtin_bit_cast(sa_bf16x8_t, u4);
}

// ---------------------------------------------------------------------------------------------
// forward
// ---------------------------------------------------------------------------------------------
constexpr int kSaT2 = 64;   // keys per tile of the forward kernel

__global__ __launch_bounds__(512) void soft_attn_fwd_kernel(SoftSeqs cs, SoftArgs a) {
    __shared__ __attribute__((aligned(16))) char s_k[2][kSaT2 * kSaRm];
    __shared__ __attribute__((aligned(16))) char s_v[2][kSaT2 * kSaCm];
    __shared__ __attribute__((aligned(16))) float s_bin[2][kSaT2];
    __shared__ __attribute__((aligned(16))) float s_bout[2][kSaT2];

    int bx, h, b;
    xcd_item(a.nx, a.Hkv, cs.n, bx, h, b);
    const int qt = a.nx - 1 - bx;  // longest rows first
    const int T = cs.ntok[b], base = cs.base[b];
    if (qt * kSaQ >= T) return;  // block-uniform
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int head = wave & 3, rb = wave >> 2;
    const int qn = lane & 31, half = lane >> 5;
    const int q0 = qt * kSaQ;
    const int i_end = min(T, q0 + kSaQ);
    const int n_tiles = (i_end + kSaT2 - 1) / kSaT2;

    sa_bf16x8_t qv[8];
    const int qi = min(q0 + rb * 32 + qn, T - 1);
    {
        const char *qp = a.q + ((size_t)(base + qi) * a.Hq + (size_t)h * kSaG + head) * kSaD * 2;
#pragma unroll
        for (int ks = 0; ks < 8; ks++) qv[ks] = *reinterpret_cast<const sa_bf16x8_t *>(qp + (ks * 16 + half * 8) * 2);
    }
    sa_f32x16_t o[4];
    // l sums the weights as the second product sees them (rounded to bf16) and normalises the
    // output; lx sums them unrounded and gives the log-sum-exp the backward pass starts from
    float m = -INFINITY, l = 0.f, lx = 0.f;
#pragma unroll
    for (int db = 0; db < 4; db++)
#pragma unroll
        for (int c = 0; c < 16; c++) o[db][c] = 0.f;

    // staging: thread -> (keys ld_key and ld_key + 32 of the tile, 16-byte chunk)
    const int ld_key = threadIdx.x >> 4, ld_dc = threadIdx.x & 15;
    const int64_t v_delta = a.v - a.k;
    uint4 kreg0, kreg1, vreg0, vreg1;
    float bin0, bout0, bin1, bout1;
    auto fetch = [&](int t) __attribute__((always_inline)) {
        const size_t row0 = (size_t)(base + min(t * kSaT2 + ld_key, T - 1)) * a.Hkv + h;
        const size_t row1 = (size_t)(base + min(t * kSaT2 + 32 + ld_key, T - 1)) * a.Hkv + h;
        const char *kp0 = a.k + row0 * (kSaD * 2) + ld_dc * 16, *kp1 = a.k + row1 * (kSaD * 2) + ld_dc * 16;
        kreg0 = *reinterpret_cast<const uint4 *>(kp0);
        kreg1 = *reinterpret_cast<const uint4 *>(kp1);
        vreg0 = *reinterpret_cast<const uint4 *>(kp0 + v_delta);
        vreg1 = *reinterpret_cast<const uint4 *>(kp1 + v_delta);
        sa_bias(a.g[row0], a.eps, bin0, bout0);
        sa_bias(a.g[row1], a.eps, bin1, bout1);
    };
    auto stage = [&](int buf) __attribute__((always_inline)) {
        sa_put_rm(s_k[buf], ld_key, ld_dc, kreg0);
        sa_put_rm(s_k[buf], ld_key + 32, ld_dc, kreg1);
        *reinterpret_cast<uint4 *>(&s_v[buf][ld_key * kSaCm + ld_dc * 16]) = vreg0;
        *reinterpret_cast<uint4 *>(&s_v[buf][(ld_key + 32) * kSaCm + ld_dc * 16]) = vreg1;
        if (ld_dc == 0) {
            s_bin[buf][ld_key] = bin0; s_bout[buf][ld_key] = bout0;
            s_bin[buf][ld_key + 32] = bin1; s_bout[buf][ld_key + 32] = bout1;
        }
    };

    fetch(0);
    stage(0);
    __syncthreads();
    for (int t = 0; t < n_tiles; t++) {
        const int buf = t & 1;
        // ---- S^T for the two halves of 32 keys ----
        sa_f32x16_t s0, s1;
#pragma unroll
        for (int c = 0; c < 16; c++) { s0[c] = 0.f; s1[c] = 0.f; }
        {
            sa_bf16x8_t ka[8];
#pragma unroll
            for (int ks = 0; ks < 8; ks++) ka[ks] = sa_get_rm(s_k[buf], qn, half, ks);
            __builtin_amdgcn_sched_barrier(0);
            if (t + 1 < n_tiles) fetch(t + 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < 8; ks++) s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qv[ks], s0, 0, 0, 0);
#pragma unroll
            for (int ks = 0; ks < 8; ks++) ka[ks] = sa_get_rm(s_k[buf], 32 + qn, half, ks);
#pragma unroll
            for (int ks = 0; ks < 8; ks++) s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qv[ks], s1, 0, 0, 0);
        }
        // register c = 4j+i of s0 (s1) holds key 8j + 4*half + i (+ 32) of the tile
        const bool far = t * kSaT2 + kSaT2 - 1 <= q0 - a.W;  // every key outside every window of the block
        float sc[32];
        float mt = -INFINITY;
#pragma unroll
        for (int hf = 0; hf < 2; hf++)
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const float4 bo4 = *reinterpret_cast<const float4 *>(&s_bout[buf][32 * hf + 8 * j + 4 * half]);
                const float bo[4] = {bo4.x, bo4.y, bo4.z, bo4.w};
                if (far) {
#pragma unroll
                    for (int i = 0; i < 4; i++) {
                        const float sv = hf ? s1[4 * j + i] : s0[4 * j + i];
                        sc[16 * hf + 4 * j + i] = fmaf(sv, a.scale_log2e, bo[i]);
                        mt = fmaxf(mt, sc[16 * hf + 4 * j + i]);
                    }
                } else {
                    const float4 bi4 = *reinterpret_cast<const float4 *>(&s_bin[buf][32 * hf + 8 * j + 4 * half]);
                    const float bi[4] = {bi4.x, bi4.y, bi4.z, bi4.w};
#pragma unroll
                    for (int i = 0; i < 4; i++) {
                        const int jg = t * kSaT2 + 32 * hf + 8 * j + 4 * half + i;
                        const float sv = hf ? s1[4 * j + i] : s0[4 * j + i];
                        const float bias = (qi - jg < a.W) ? bi[i] : bo[i];
                        const float x = (jg <= qi) ? fmaf(sv, a.scale_log2e, bias) : -INFINITY;
                        sc[16 * hf + 4 * j + i] = x;
                        mt = fmaxf(mt, x);
                    }
                }
            }
        mt = fmaxf(mt, __shfl_xor(mt, 32));
        const float mnew = fmaxf(m, mt);
        const float msafe = mnew == -INFINITY ? 0.f : mnew;
        const float corr = __builtin_amdgcn_exp2f(m - msafe);
        uint32_t pb[16];
        float ps = 0.f, px = 0.f;
        const sa_bf16x2_t ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
        for (int c = 0; c < 16; c++) {
            const float p0 = __builtin_amdgcn_exp2f(sc[2 * c] - msafe), p1 = __builtin_amdgcn_exp2f(sc[2 * c + 1] - msafe);
            px += p0 + p1;
            pb[c] = sa_pack(p0, p1);
            ps = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(sa_bf16x2_t, pb[c]), ones, ps, false);
        }
        l = l * corr + ps;
        lx = lx * corr + px;
        if (__builtin_amdgcn_ballot_w64(mnew > m) != 0) {
#pragma unroll
            for (int db = 0; db < 4; db++)
#pragma unroll
                for (int c = 0; c < 16; c++) o[db][c] *= corr;
        }
        m = mnew;
        // ---- O^T += V^T P^T, four steps of 16 keys ----
#pragma unroll
        for (int t2 = 0; t2 < 4; t2++) {
            const uint4 p4 = make_uint4(pb[4 * t2], pb[4 * t2 + 1], pb[4 * t2 + 2], pb[4 * t2 + 3]);
            const sa_bf16x8_t pbv = __builtin_bit_cast(sa_bf16x8_t, p4);
#pragma unroll
            for (int db = 0; db < 4; db++)
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sa_get_cols<kSaCm>(s_v[buf], lane, db, 16 * t2), pbv, o[db], 0, 0, 0);
        }
        if (t + 1 < n_tiles) stage(buf ^ 1);
        __syncthreads();
    }
    // register c = 4j+i of o[db] is d = 32*db + 8j + 4*half + i
    const int i = q0 + rb * 32 + qn;
    const float lt = l + __shfl_xor(l, 32), lxt = lx + __shfl_xor(lx, 32);
    if (i < T) {
        const float inv = 1.0f / lt;
        const size_t orow = (size_t)(base + i) * a.Hq + (size_t)h * kSaG + head;
        float *op = a.out + orow * kSaD;
#pragma unroll
        for (int db = 0; db < 4; db++)
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const float4 w4 = make_float4(o[db][4 * j] * inv, o[db][4 * j + 1] * inv, o[db][4 * j + 2] * inv,
                                              o[db][4 * j + 3] * inv);
                *reinterpret_cast<float4 *>(op + 32 * db + 8 * j + 4 * half) = w4;
            }
        if (half == 0) a.lse[orow] = (m + __log2f(lxt)) * 0.6931471805599453f;
    }
}

// ---------------------------------------------------------------------------------------------
// backward, step 0: D_i = dO_i . O_i   (32 lanes per row)
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void soft_attn_rowdot_kernel(int64_t n_rows, const char *dout, const float *out,
                                                               float *rowdot) {
    const int64_t r = (int64_t)blockIdx.x * 8 + (threadIdx.x >> 5);
    const int sub = threadIdx.x & 31;
    float acc = 0.f;
    if (r < n_rows) {
        const uint2 d2 = *reinterpret_cast<const uint2 *>(dout + (size_t)r * kSaD * 2 + sub * 8);
        const float4 o4 = *reinterpret_cast<const float4 *>(out + (size_t)r * kSaD + sub * 4);
        acc = __uint_as_float(d2.x << 16) * o4.x + __uint_as_float(d2.x & 0xffff0000u) * o4.y +
              __uint_as_float(d2.y << 16) * o4.z + __uint_as_float(d2.y & 0xffff0000u) * o4.w;
    }
    acc = group_sum<32>(acc);
    if (r < n_rows && sub == 0) rowdot[r] = acc;
}

// ---------------------------------------------------------------------------------------------
// backward, dQ: columns of every tile are this wave's 32 queries
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void soft_attn_bwd_dq_kernel(SoftSeqs cs, SoftArgs a) {
    __shared__ __attribute__((aligned(16))) char s_k[2][kSaT * kSaRm];
    __shared__ __attribute__((aligned(16))) char s_kc[2][kSaT * kSaCm];  // the same tile at the stride of column reads
    __shared__ __attribute__((aligned(16))) char s_v[2][kSaT * kSaRm];
    __shared__ __attribute__((aligned(16))) float s_bin[2][kSaT];
    __shared__ __attribute__((aligned(16))) float s_bout[2][kSaT];

    int bx, h, b;
    xcd_item(a.nx, a.Hkv, cs.n, bx, h, b);
    const int qt = a.nx - 1 - bx;
    const int T = cs.ntok[b], base = cs.base[b];
    if (qt * kSaQ >= T) return;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int head = wave & 3, rb = wave >> 2;
    const int qn = lane & 31, half = lane >> 5;
    const int q0 = qt * kSaQ;
    const int i_end = min(T, q0 + kSaQ);
    const int n_tiles = (i_end + kSaT - 1) / kSaT;

    const int qi = min(q0 + rb * 32 + qn, T - 1);
    const size_t qrow = (size_t)(base + qi) * a.Hq + (size_t)h * kSaG + head;
    sa_bf16x8_t qv[8], dov[8];
    {
        const char *qp = a.q + qrow * kSaD * 2, *dp = a.dout + qrow * kSaD * 2;
#pragma unroll
        for (int ks = 0; ks < 8; ks++) {
            qv[ks] = *reinterpret_cast<const sa_bf16x8_t *>(qp + (ks * 16 + half * 8) * 2);
            dov[ks] = *reinterpret_cast<const sa_bf16x8_t *>(dp + (ks * 16 + half * 8) * 2);
        }
    }
    const float lse2 = a.lse[qrow] * 1.4426950408889634f;
    const float Di = a.rowdot[qrow];
    sa_f32x16_t dq[4];
#pragma unroll
    for (int db = 0; db < 4; db++)
#pragma unroll
        for (int c = 0; c < 16; c++) dq[db][c] = 0.f;

    const int ld_key = threadIdx.x >> 4, ld_dc = threadIdx.x & 15;  // thread -> (key of the tile, 16-byte chunk)
    const int64_t v_delta = a.v - a.k;
    // two sets of staging registers: a tile is requested two iterations before it is multiplied
    struct StReg { uint4 kreg, vreg; float bin_reg, bout_reg; };
    StReg r0, r1;
    auto fetch = [&](int t, StReg &r) __attribute__((always_inline)) {
        const size_t row = (size_t)(base + min(t * kSaT + ld_key, T - 1)) * a.Hkv + h;
        const char *kp = a.k + row * (kSaD * 2) + ld_dc * 16;
        r.kreg = *reinterpret_cast<const uint4 *>(kp);
        r.vreg = *reinterpret_cast<const uint4 *>(kp + v_delta);
        sa_bias(a.g[row], a.eps, r.bin_reg, r.bout_reg);
    };
    auto stage = [&](int buf, const StReg &r) __attribute__((always_inline)) {
        sa_put_rm(s_k[buf], ld_key, ld_dc, r.kreg);
        *reinterpret_cast<uint4 *>(&s_kc[buf][ld_key * kSaCm + ld_dc * 16]) = r.kreg;
        sa_put_rm(s_v[buf], ld_key, ld_dc, r.vreg);
        if (ld_dc == 0) { s_bin[buf][ld_key] = r.bin_reg; s_bout[buf][ld_key] = r.bout_reg; }
    };

    fetch(0, r0);
    stage(0, r0);
    if (n_tiles > 1) fetch(1, r1);
    __syncthreads();
    // one iteration: tile t is multiplied, tile t+2 is requested into rf, tile t+1 goes from rs to LDS
    auto body = [&](int t, StReg &rf, const StReg &rs) __attribute__((always_inline)) {
        const int buf = t & 1;
        sa_bf16x8_t ka[8];
#pragma unroll
        for (int ks = 0; ks < 8; ks++) ka[ks] = sa_get_rm(s_k[buf], qn, half, ks);
        __builtin_amdgcn_sched_barrier(0);
        if (t + 2 < n_tiles) fetch(t + 2, rf);
        __builtin_amdgcn_sched_barrier(0);
        sa_f32x16_t s, dp;
#pragma unroll
        for (int c = 0; c < 16; c++) { s[c] = 0.f; dp[c] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < 8; ks++) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qv[ks], s, 0, 0, 0);
#pragma unroll
        for (int ks = 0; ks < 8; ks++) ka[ks] = sa_get_rm(s_v[buf], qn, half, ks);
#pragma unroll
        for (int ks = 0; ks < 8; ks++) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], dov[ks], dp, 0, 0, 0);
        // dS^T = P^T (dP^T - D_i), rounded to bf16 for the last product
        uint32_t db_[8];
        const bool far = t * kSaT + kSaT - 1 <= q0 - a.W;  // every key outside every window of the block: no mask, one bias
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const float4 bo4 = *reinterpret_cast<const float4 *>(&s_bout[buf][8 * j + 4 * half]);
            const float bo[4] = {bo4.x, bo4.y, bo4.z, bo4.w};
            float ds[4];
            if (far) {
#pragma unroll
                for (int i = 0; i < 4; i++)
                    ds[i] = __builtin_amdgcn_exp2f(fmaf(s[4 * j + i], a.scale_log2e, bo[i] - lse2)) * (dp[4 * j + i] - Di);
            } else {
                const float4 bi4 = *reinterpret_cast<const float4 *>(&s_bin[buf][8 * j + 4 * half]);
                const float bi[4] = {bi4.x, bi4.y, bi4.z, bi4.w};
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const int jg = t * kSaT + 8 * j + 4 * half + i;
                    const float bias = (qi - jg < a.W) ? bi[i] : bo[i];
                    const float x = (jg <= qi) ? fmaf(s[4 * j + i], a.scale_log2e, bias) - lse2 : -INFINITY;
                    ds[i] = __builtin_amdgcn_exp2f(x) * (dp[4 * j + i] - Di);
                }
            }
            db_[2 * j] = sa_pack(ds[0], ds[1]);
            db_[2 * j + 1] = sa_pack(ds[2], ds[3]);
        }
#pragma unroll
        for (int t2 = 0; t2 < 2; t2++) {
            const uint4 p4 = make_uint4(db_[4 * t2], db_[4 * t2 + 1], db_[4 * t2 + 2], db_[4 * t2 + 3]);
            const sa_bf16x8_t dsv = __builtin_bit_cast(sa_bf16x8_t, p4);
#pragma unroll
            for (int db = 0; db < 4; db++)
                dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sa_get_cols<kSaCm>(s_kc[buf], lane, db, 16 * t2), dsv, dq[db], 0, 0, 0);
        }
        if (t + 1 < n_tiles) stage(buf ^ 1, rs);
        __syncthreads();
    };
    {
        int t = 0;
        for (; t + 1 < n_tiles; t += 2) {
            body(t, r0, r1);
            body(t + 1, r1, r0);
        }
        if (t < n_tiles) body(t, r0, r1);
    }
    const int i = q0 + rb * 32 + qn;
    if (i < T) {
        float *op = a.dq + qrow * kSaD;
#pragma unroll
        for (int db = 0; db < 4; db++)
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const float4 w4 = make_float4(dq[db][4 * j] * a.scale, dq[db][4 * j + 1] * a.scale,
                                              dq[db][4 * j + 2] * a.scale, dq[db][4 * j + 3] * a.scale);
                *reinterpret_cast<float4 *>(op + 32 * db + 8 * j + 4 * half) = w4;
            }
    }
}

// ---------------------------------------------------------------------------------------------
// backward, dK / dV / dg: columns of every tile are this wave's 32 keys
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void soft_attn_bwd_dkv_kernel(SoftSeqs cs, SoftArgs a) {
    // Role 0 works on tile `it` while role 1 works on tile it-1 (it gets P of that tile from role 0
    // through LDS, written one iteration earlier): one barrier per iteration, and the two waves of
    // a SIMD never wait for each other inside one.  What role 0 reads needs two buffers (in use,
    // being staged), what role 1 reads needs three (in use, waiting, being staged).
    __shared__ __attribute__((aligned(16))) char s_q[2][kSaT * kSaRm];     // role 0: rows (S = Q K^T)
    __shared__ __attribute__((aligned(16))) char s_doc[2][kSaT * kSaCm];   // role 0: columns (dV^T += dO^T P)
    __shared__ __attribute__((aligned(16))) char s_do[3][kSaT * kSaRm];    // role 1: rows (dP = dO V^T)
    __shared__ __attribute__((aligned(16))) char s_qc[3][kSaT * kSaCm];    // role 1: columns (dK^T += Q^T dS)
    __shared__ __attribute__((aligned(16))) float s_lse[2][kSaT];
    __shared__ __attribute__((aligned(16))) float s_dd[3][kSaT];
    __shared__ float s_p[2][4][16][64];  // P of a (32 keys x 32 queries) tile per key sub-tile, lane-private slots

    int kbk, h, b;  // early key blocks have the most queries: first
    xcd_item(a.nx, a.Hkv, cs.n, kbk, h, b);
    const int T = cs.ntok[b], base = cs.base[b];
    const int j0 = kbk * kSaKB;
    if (j0 >= T) return;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int kb = wave & 3, role = wave >> 2;
    const int qn = lane & 31, half = lane >> 5;
    const int jg = j0 + kb * 32 + qn;        // this lane's key
    const int jc = min(jg, T - 1);
    const size_t krow = (size_t)(base + jc) * a.Hkv + h;

    // the block's own rows: K for role 0, V for role 1, as the N side of a product over d
    sa_bf16x8_t own[8];
    {
        const char *p = (role == 0 ? a.k : a.v) + krow * kSaD * 2;
#pragma unroll
        for (int ks = 0; ks < 8; ks++) own[ks] = *reinterpret_cast<const sa_bf16x8_t *>(p + (ks * 16 + half * 8) * 2);
    }
    const float gj = a.g[krow];
    float b_in, b_out;
    sa_bias(gj, a.eps, b_in, b_out);
    const bool follows_in = gj > 1.0f, follows_out = gj > 0.0f;  // where m_ij is g_j rather than the indicator
    sa_f32x16_t acc[4];  // role 0: dV^T, role 1: dK^T ; rows d, columns keys
#pragma unroll
    for (int db = 0; db < 4; db++)
#pragma unroll
        for (int c = 0; c < 16; c++) acc[db][c] = 0.f;
    float dg_acc = 0.f;

    // streamed tiles: 32 queries of one query head; iteration it = (query tile, head)
    const int qt_first = j0 / kSaT, n_qt = (T + kSaT - 1) / kSaT;
    const int n_it = (n_qt - qt_first) * kSaG;
    const int ld_row = threadIdx.x >> 4, ld_dc = threadIdx.x & 15;  // thread -> (row of the tile, 16-byte chunk)
    // two sets of staging registers: the loads of a tile are issued two iterations before the
    // tile is multiplied (one iteration is shorter than the latency of a load under this traffic)
    struct StReg { uint4 qreg, doreg; float lse_reg, dd_reg; };
    StReg r0, r1;
    auto fetch = [&](int it, StReg &r) __attribute__((always_inline)) {
        const int qt = qt_first + it / kSaG, hd = it % kSaG;
        const int idx = qt * kSaT + ld_row;
        const size_t row = (size_t)(base + min(idx, T - 1)) * a.Hq + (size_t)h * kSaG + hd;
        r.qreg = *reinterpret_cast<const uint4 *>(a.q + row * (kSaD * 2) + ld_dc * 16);
        r.doreg = *reinterpret_cast<const uint4 *>(a.dout + row * (kSaD * 2) + ld_dc * 16);
        const bool real = idx < T;  // a row past the end gets weight exp2(-inf) = 0
        r.lse_reg = real ? a.lse[row] * 1.4426950408889634f : INFINITY;
        r.dd_reg = real ? a.rowdot[row] : 0.f;
    };
    auto stage = [&](int b2, int b3, const StReg &r) __attribute__((always_inline)) {
        sa_put_rm(s_q[b2], ld_row, ld_dc, r.qreg);
        sa_put_rm(s_do[b3], ld_row, ld_dc, r.doreg);
        *reinterpret_cast<uint4 *>(&s_qc[b3][ld_row * kSaCm + ld_dc * 16]) = r.qreg;
        *reinterpret_cast<uint4 *>(&s_doc[b2][ld_row * kSaCm + ld_dc * 16]) = r.doreg;
        if (ld_dc == 0) { s_lse[b2][ld_row] = r.lse_reg; s_dd[b3][ld_row] = r.dd_reg; }
    };

    fetch(0, r0);
    stage(0, 0, r0);
    fetch(1, r1);  // n_it >= 4
    __syncthreads();
    int b3 = 0;  // it % 3
    // one iteration: role 0 multiplies tile `it`, role 1 tile it-1; tile it+2 is requested into rf,
    // tile it+1 goes from rs to LDS
    auto body = [&](int it, StReg &rf, const StReg &rs) __attribute__((always_inline)) {
        const int b3p = b3 == 0 ? 2 : b3 - 1, b3n = b3 == 2 ? 0 : b3 + 1;
        const int mine = role == 0 ? it : it - 1;               // the tile this wave multiplies
        const bool active = role == 0 ? it < n_it : it >= 1;    // wave-uniform
        const int i0 = (qt_first + mine / kSaG) * kSaT;         // first query of that tile
        // first product: rows = queries of the tile, columns = this wave's keys
        const char *rm = role == 0 ? s_q[it & 1] : s_do[b3p];
        sa_bf16x8_t fa[8];
        if (active) {
#pragma unroll
            for (int ks = 0; ks < 8; ks++) fa[ks] = sa_get_rm(rm, qn, half, ks);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (it + 2 < n_it) fetch(it + 2, rf);
        __builtin_amdgcn_sched_barrier(0);
        if (active) {
            sa_f32x16_t x;
#pragma unroll
            for (int c = 0; c < 16; c++) x[c] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ks++) x = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks], own[ks], x, 0, 0, 0);
            // register c = 4j+i of a lane holds query i0 + 8j + 4*half + i
            uint32_t pk[8];
            // wave-uniform: every query of the tile follows every key of this wave by at least the window, so no
            // pair is masked and every bias is the one outside the window (nearly all tiles of a long sequence)
            const bool interior = i0 - (j0 + kb * 32 + 31) >= a.W;
            if (role == 0 && interior) {
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    const float4 l4 = *reinterpret_cast<const float4 *>(&s_lse[it & 1][8 * j + 4 * half]);
                    const float ls[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
                    for (int i = 0; i < 4; i++) {
                        x[4 * j + i] = __builtin_amdgcn_exp2f(fmaf(x[4 * j + i], a.scale_log2e, b_out - ls[i]));
                        s_p[it & 1][kb][4 * j + i][lane] = x[4 * j + i];
                    }
                }
#pragma unroll
                for (int c = 0; c < 8; c++) pk[c] = sa_pack(x[2 * c], x[2 * c + 1]);
            } else if (role == 0) {
                // P = exp2(S * scale + bias - lse); a copy goes to the partner wave through LDS
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    const float4 l4 = *reinterpret_cast<const float4 *>(&s_lse[it & 1][8 * j + 4 * half]);
                    const float ls[4] = {l4.x, l4.y, l4.z, l4.w};
#pragma unroll
                    for (int i = 0; i < 4; i++) {
                        const int ig = i0 + 8 * j + 4 * half + i;
                        const float bias = (ig - jg < a.W) ? b_in : b_out;
                        const float e = (jg <= ig) ? fmaf(x[4 * j + i], a.scale_log2e, bias) - ls[i] : -INFINITY;
                        x[4 * j + i] = __builtin_amdgcn_exp2f(e);
                        s_p[it & 1][kb][4 * j + i][lane] = x[4 * j + i];
                    }
                }
#pragma unroll
                for (int c = 0; c < 8; c++) pk[c] = sa_pack(x[2 * c], x[2 * c + 1]);
            } else if (interior) {
                float dsum = 0.f;
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    const float4 d4 = *reinterpret_cast<const float4 *>(&s_dd[b3p][8 * j + 4 * half]);
                    const float dd[4] = {d4.x, d4.y, d4.z, d4.w};
                    float ds[4];
#pragma unroll
                    for (int i = 0; i < 4; i++) {
                        ds[i] = s_p[mine & 1][kb][4 * j + i][lane] * (x[4 * j + i] - dd[i]);
                        dsum += ds[i];
                    }
                    pk[2 * j] = sa_pack(ds[0], ds[1]);
                    pk[2 * j + 1] = sa_pack(ds[2], ds[3]);
                }
                dg_acc += follows_out ? dsum : 0.f;
            } else {
                // dS = P (dP - D_i); the part of it where m_ij follows g_j adds up to dg_j (g_j + eps)
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    const float4 d4 = *reinterpret_cast<const float4 *>(&s_dd[b3p][8 * j + 4 * half]);
                    const float dd[4] = {d4.x, d4.y, d4.z, d4.w};
                    float ds[4];
#pragma unroll
                    for (int i = 0; i < 4; i++) {
                        const int ig = i0 + 8 * j + 4 * half + i;
                        ds[i] = s_p[mine & 1][kb][4 * j + i][lane] * (x[4 * j + i] - dd[i]);
                        const bool follows = (ig - jg < a.W) ? follows_in : follows_out;
                        dg_acc += follows ? ds[i] : 0.f;
                    }
                    pk[2 * j] = sa_pack(ds[0], ds[1]);
                    pk[2 * j + 1] = sa_pack(ds[2], ds[3]);
                }
            }
            // second product: rows = d, columns = keys, contraction over the 32 queries (the rows of
            // the staged tile, read column-wise)
            const char *tr = role == 0 ? s_doc[it & 1] : s_qc[b3p];
#pragma unroll
            for (int t2 = 0; t2 < 2; t2++) {
                const uint4 p4 = make_uint4(pk[4 * t2], pk[4 * t2 + 1], pk[4 * t2 + 2], pk[4 * t2 + 3]);
                const sa_bf16x8_t pv = __builtin_bit_cast(sa_bf16x8_t, p4);
#pragma unroll
                for (int db = 0; db < 4; db++)
                    acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sa_get_cols<kSaCm>(tr, lane, db, 16 * t2), pv, acc[db], 0, 0, 0);
            }
        }
        if (it + 1 < n_it) stage((it + 1) & 1, b3n, rs);
        __syncthreads();
        b3 = b3n;
    };
    for (int it = 0; it <= n_it; it += 2) {  // n_it is a multiple of 4; one more turn for role 1's last tile
        body(it, r0, r1);
        if (it + 1 <= n_it) body(it + 1, r1, r0);
    }
    if (jg < T) {
        float *op = (role == 0 ? a.dv : a.dk) + krow * kSaD;
        const float f = role == 0 ? 1.0f : a.scale;
#pragma unroll
        for (int db = 0; db < 4; db++)
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const float4 w4 = make_float4(acc[db][4 * j] * f, acc[db][4 * j + 1] * f, acc[db][4 * j + 2] * f,
                                              acc[db][4 * j + 3] * f);
                *reinterpret_cast<float4 *>(op + 32 * db + 8 * j + 4 * half) = w4;
            }
    }
    if (role == 1) {
        const float tot = dg_acc + __shfl_xor(dg_acc, 32);
        if (half == 0 && jg < T) a.dg[krow] = follows_out ? tot / (gj + a.eps) : 0.f;
    }
}

// ---------------------------------------------------------------------------------------------
static bool soft_fill(SoftSeqs &cs, int n_seqs, const int32_t *n_tokens, int *max_t, int64_t *total) {
    if (n_seqs < 0 || n_seqs > kMaxCallSeqs) return false;
    cs.n = n_seqs;
    int64_t tot = 0;
    int mx = 0;
    for (int b = 0; b < n_seqs; b++) {
        if (n_tokens[b] < 0) return false;
        cs.ntok[b] = n_tokens[b];
        cs.base[b] = (int32_t)tot;
        tot += n_tokens[b];
        if (tot >= ((int64_t)1 << 24)) return false;  // keeps every packed row index far inside 32 bits
        mx = max(mx, n_tokens[b]);
    }
    *max_t = mx;
    *total = tot;
    return true;
}

size_t soft_attn_ws_bytes(int64_t total_tokens, int n_q_heads) {
    return (size_t)((total_tokens * n_q_heads * 4 + 255) / 256) * 256;
}

hipError_t launch_soft_attn_fwd(int n_seqs, const int32_t *n_tokens, int Hq, int Hkv, int d, int W,
                                const void *q, const void *k, const void *v, const float *g, float scale,
                                float eps, float *out, float *lse, hipStream_t st) {
    if (d != kSaD || Hq != Hkv * kSaG) return hipErrorNotSupported;
    SoftSeqs cs;
    int max_t;
    int64_t total;
    if (!soft_fill(cs, n_seqs, n_tokens, &max_t, &total)) return hipErrorInvalidValue;
    if (max_t == 0) return hipSuccess;
    SoftArgs a = {};
    a.Hq = Hq; a.Hkv = Hkv; a.W = W;
    a.scale = scale; a.scale_log2e = scale * 1.4426950408889634f; a.eps = eps;
    a.q = (const char *)q; a.k = (const char *)k; a.v = (const char *)v; a.g = g;
    a.out = out; a.lse = lse;
    a.nx = (max_t + kSaQ - 1) / kSaQ;
    hipLaunchKernelGGL(soft_attn_fwd_kernel, dim3(a.nx * Hkv * n_seqs), dim3(512), 0, st, cs, a);
    return hipGetLastError();
}

hipError_t launch_soft_attn_bwd(int n_seqs, const int32_t *n_tokens, int Hq, int Hkv, int d, int W,
                                const void *q, const void *k, const void *v, const float *g, float scale,
                                float eps, const float *out, const float *lse, const void *dout, float *dq,
                                float *dk, float *dv, float *dg, void *ws, hipStream_t st) {
    if (d != kSaD || Hq != Hkv * kSaG) return hipErrorNotSupported;
    SoftSeqs cs;
    int max_t;
    int64_t total;
    if (!soft_fill(cs, n_seqs, n_tokens, &max_t, &total)) return hipErrorInvalidValue;
    if (max_t == 0) return hipSuccess;
    SoftArgs a = {};
    a.Hq = Hq; a.Hkv = Hkv; a.W = W;
    a.scale = scale; a.scale_log2e = scale * 1.4426950408889634f; a.eps = eps;
    a.q = (const char *)q; a.k = (const char *)k; a.v = (const char *)v; a.g = g;
    a.out = const_cast<float *>(out); a.lse = const_cast<float *>(lse);
    a.dout = (const char *)dout;
    a.rowdot = (float *)ws;
    a.dq = dq; a.dk = dk; a.dv = dv; a.dg = dg;
    const int64_t n_rows = total * Hq;
    hipLaunchKernelGGL(soft_attn_rowdot_kernel, dim3((unsigned)((n_rows + 7) / 8)), dim3(256), 0, st, n_rows,
                       a.dout, out, a.rowdot);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    a.nx = (max_t + kSaQ - 1) / kSaQ;
    hipLaunchKernelGGL(soft_attn_bwd_dq_kernel, dim3(a.nx * Hkv * n_seqs), dim3(512), 0, st, cs, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    a.nx = (max_t + kSaKB - 1) / kSaKB;
    hipLaunchKernelGGL(soft_attn_bwd_dkv_kernel, dim3(a.nx * Hkv * n_seqs), dim3(512), 0, st, cs, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Sparsity term of the training objective (Sec. 3.3): sum over the given scores of
// (g + g (1 - g)) / n_total and its derivative (2 - 2 g) / n_total.  Two launches with a fixed
// order of additions (per-thread strided sums, block tree, then one thread over the blocks in
// double), so the value repeats bit for bit.
// ---------------------------------------------------------------------------------------------
constexpr int kSpBlocks = 1024;

__global__ __launch_bounds__(256) void sparsity_partial_kernel(const float *g, int64_t n, float inv_n, float *dg,
                                                               float *partial) {
    __shared__ float s_red[256];
    float acc = 0.f;
    for (int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x; x < n; x += (int64_t)gridDim.x * 256) {
        const float v = g[x];
        acc += v + v * (1.0f - v);
        if (dg) dg[x] = (2.0f - 2.0f * v) * inv_n;
    }
    s_red[threadIdx.x] = acc;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) s_red[threadIdx.x] += s_red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[blockIdx.x] = s_red[0];
}

__global__ void sparsity_final_kernel(const float *partial, int nb, double inv_n, float *loss) {
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    double t = 0.0;
    for (int i = 0; i < nb; i++) t += (double)partial[i];
    *loss = (float)(t * inv_n);
}

size_t sparsity_ws_bytes() { return kSpBlocks * sizeof(float); }

hipError_t launch_sparsity_loss(const float *g, int64_t n, int64_t n_total, float *loss, float *dg, void *ws,
                                hipStream_t st) {
    const int nb = (int)std::min<int64_t>(kSpBlocks, std::max<int64_t>(1, (n + 255) / 256));
    const double inv = 1.0 / (double)n_total;
    hipLaunchKernelGGL(sparsity_partial_kernel, dim3(nb), dim3(256), 0, st, g, n, (float)inv, dg, (float *)ws);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(sparsity_final_kernel, dim3(1), dim3(64), 0, st, (const float *)ws, nb, inv, loss);
    return hipGetLastError();
}

}  // namespace wgkv
