// Chunked-prefill attention under the vertical-slash mask (Sec. 4.2 mask equation)
// on the gfx950 matrix cores.
//
// Query i of the chunk (position t0+i) of a kv head's group sees
//   - every entry of the head's global cache (admitted tokens older than the window),
//   - ring positions j in [t0-W, t0) with  pos_i - j < W  or stored g_j >= tau,
//   - chunk keys j <= i with  i - j < W  or g_j >= tau,
// which is exactly M_ij restricted to what is still known about the past: tokens
// that were neither admitted nor inside the window are gone (Sec. 4.2, "Initial
// cache population") and are invisible under M_ij anyway.
//
// One block owns 64 chunk positions of one (sequence, kv head); its four waves are
// the four query heads of the group, so a K/V tile staged in LDS feeds all of them.
// Everything is computed transposed, S^T = K Q^T and O^T = V^T P^T with
// v_mfma_f32_32x32x16_bf16: a lane then owns one query column, so the running max,
// the denominator and the rescale factor are plain per-lane scalars, and the
// probabilities leave the first product already in the operand layout of the second.
#include <climits>

#include "wgkv_dev.h"

namespace wgkv {

typedef __attribute__((ext_vector_type(8))) __bf16 pf_bf16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 pf_bf16x2_t;
typedef __attribute__((ext_vector_type(16))) float pf_f32x16_t;

constexpr int kPfD = 128;         // head_dim
constexpr int kPfQ = 64;          // chunk positions per block (2 row blocks of 32)
constexpr int kPfKT = 32;         // keys per tile
constexpr int kPfKStride = 272;   // bytes per key row of the K tile in LDS (256 + 16 pad)
constexpr int kPfVStride = 72;    // bytes per d row of the transposed V tile (64 + 8 pad)

struct PrefillAttnArgs {
    int layer;
    float tau;
    float scale_log2e;
    const char *q, *k, *v;  // chunk tensors, bf16
    const float *g;         // chunk scores
    float *out;
};

__device__ __forceinline__ uint32_t pf_pack(float lo, float hi) {
    pf_bf16x2_t t = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, t);
}

__global__ __launch_bounds__(256) void attend_prefill_kernel(View pv, CallSeqs cs, PrefillAttnArgs a) {
    __shared__ __attribute__((aligned(16))) char s_k[2][kPfKT * kPfKStride];
    __shared__ __attribute__((aligned(16))) char s_vt[2][kPfD * kPfVStride];
    __shared__ __attribute__((aligned(16))) int s_lo[2][kPfKT];
    __shared__ __attribute__((aligned(16))) int s_hi[2][kPfKT];

    const int b = blockIdx.z, h = blockIdx.y, qt = blockIdx.x;
    const int T = cs.ntok[b], t0 = cs.t0[b], base = cs.base[b];
    if (qt * kPfQ >= T) return;  // block-uniform
    const int sid = cs.sid[b];
    const int um = unit_meta(pv, sid, a.layer, h);
    const int G = 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int qn = lane & 31, half = lane >> 5;
    const int gl = pv.global_len[um];
    const int w_eff = min(pv.W, t0);              // ring entries that exist
    const int i_end = min(T, qt * kPfQ + kPfQ);   // chunk keys this block can see: [0, i_end)
    const int n_g = (gl + kPfKT - 1) / kPfKT, n_r = (w_eff + kPfKT - 1) / kPfKT;
    const int n_c = (i_end + kPfKT - 1) / kPfKT;
    const int n_tiles = n_g + n_r + n_c;

    // ---- Q^T operand: this lane's query of each row block, all 8 d-slices of 16 ----
    pf_bf16x8_t qv[2][8];
    int qpos[2];
#pragma unroll
    for (int rb = 0; rb < 2; rb++) {
        const int i = min(qt * kPfQ + rb * 32 + qn, T - 1);
        qpos[rb] = t0 + i;
        const char *qp = a.q + ((size_t)(base + i) * pv.Hq + (size_t)h * G + wave) * kPfD * 2;
#pragma unroll
        for (int ks = 0; ks < 8; ks++)
            qv[rb][ks] = *reinterpret_cast<const pf_bf16x8_t *>(qp + (ks * 16 + half * 8) * 2);
    }

    pf_f32x16_t o[2][4];
    float m[2], l[2];
#pragma unroll
    for (int rb = 0; rb < 2; rb++) {
        m[rb] = -INFINITY;
        l[rb] = 0.f;
#pragma unroll
        for (int db = 0; db < 4; db++)
#pragma unroll
            for (int c = 0; c < 16; c++) o[rb][db][c] = 0.f;
    }

    // ---- staging of a key tile: thread -> (key, 16-byte d chunk), two passes ----
    const int ld_key = threadIdx.x >> 4, ld_dc = threadIdx.x & 15;
    uint4 kreg[2], vreg[2];
    int lo_reg[2], hi_reg[2];
    auto fetch = [&](int t) {
#pragma unroll
        for (int p = 0; p < 2; p++) {
            const int key = ld_key + 16 * p;
            const char *kp, *vp;
            int lo = INT_MAX, hi = INT_MAX;  // invisible unless shown otherwise
            if (t < n_g) {                   // global cache: visible to every query
                const int idx = t * kPfKT + key, idc = min(idx, gl - 1);
                const char *pg = page_ptr(pv, pv.global_pt[(size_t)um * pv.maxgp + (idc >> pv.logP)]) +
                                 (size_t)(idc & (pv.P - 1)) * (kPfD * 2);
                kp = pg;
                vp = pg + pv.v_off;
                if (idx < gl) lo = INT_MIN;
            } else if (t < n_g + n_r) {      // ring, oldest position first
                const int idx = (t - n_g) * kPfKT + key, idc = min(idx, w_eff - 1);
                const int pos = t0 - w_eff + idc, slot = pos % pv.W;
                const char *pg = page_ptr(pv, pv.local_pt[(size_t)um * pv.nlp + (slot >> pv.logP)]) +
                                 (size_t)(slot & (pv.P - 1)) * (kPfD * 2);
                kp = pg;
                vp = pg + pv.v_off;
                if (idx < w_eff) {
                    lo = pos;
                    hi = (pv.ring_g[(size_t)um * pv.W + slot] >= a.tau) ? INT_MAX : pos + pv.W - 1;
                }
            } else {                         // this chunk
                const int idx = (t - n_g - n_r) * kPfKT + key, idc = min(idx, T - 1);
                const size_t row = (size_t)(base + idc) * pv.Hkv + h;
                kp = a.k + row * (kPfD * 2);
                vp = a.v + row * (kPfD * 2);
                if (idx < T) {
                    lo = t0 + idx;
                    hi = (a.g[row] >= a.tau) ? INT_MAX : t0 + idx + pv.W - 1;
                }
            }
            kreg[p] = *reinterpret_cast<const uint4 *>(kp + ld_dc * 16);
            vreg[p] = *reinterpret_cast<const uint4 *>(vp + ld_dc * 16);
            lo_reg[p] = lo;
            hi_reg[p] = hi;
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int p = 0; p < 2; p++) {
            const int key = ld_key + 16 * p;
            *reinterpret_cast<uint4 *>(&s_k[buf][key * kPfKStride + ld_dc * 16]) = kreg[p];
            const uint32_t w[4] = {vreg[p].x, vreg[p].y, vreg[p].z, vreg[p].w};
#pragma unroll
            for (int e = 0; e < 8; e++) {  // transposed: [d][key]
                const unsigned short x = (unsigned short)((e & 1) ? (w[e >> 1] >> 16) : (w[e >> 1] & 0xffffu));
                *reinterpret_cast<unsigned short *>(&s_vt[buf][(ld_dc * 8 + e) * kPfVStride + key * 2]) = x;
            }
            if (ld_dc == 0) { s_lo[buf][key] = lo_reg[p]; s_hi[buf][key] = hi_reg[p]; }
        }
    };

    fetch(0);
    stage(0);
    __syncthreads();

    for (int t = 0; t < n_tiles; t++) {
        const int buf = t & 1;
        if (t + 1 < n_tiles) fetch(t + 1);  // in flight while this tile is multiplied

        // ---- S^T = K Q^T : rows = keys of the tile, columns = this wave's queries ----
        pf_f32x16_t s[2];
#pragma unroll
        for (int rb = 0; rb < 2; rb++)
#pragma unroll
            for (int c = 0; c < 16; c++) s[rb][c] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ks++) {
            const pf_bf16x8_t ka =
                *reinterpret_cast<const pf_bf16x8_t *>(&s_k[buf][qn * kPfKStride + (ks * 16 + half * 8) * 2]);
            s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qv[0][ks], s[0], 0, 0, 0);
            s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qv[1][ks], s[1], 0, 0, 0);
        }
        // register c = 4j+i of a lane holds key 8j + 4*half + i of the tile
        const bool plain = (t < n_g) && ((t + 1) * kPfKT <= gl);  // full tile of the global cache: no mask
        uint32_t pb[2][8];
#pragma unroll
        for (int rb = 0; rb < 2; rb++) {
            float sc[16];
            float mt = -INFINITY;
#pragma unroll
            for (int j = 0; j < 4; j++) {
                int4 lo4 = make_int4(INT_MIN, INT_MIN, INT_MIN, INT_MIN), hi4 = make_int4(INT_MAX, INT_MAX, INT_MAX, INT_MAX);
                if (!plain) {
                    lo4 = *reinterpret_cast<const int4 *>(&s_lo[buf][8 * j + 4 * half]);
                    hi4 = *reinterpret_cast<const int4 *>(&s_hi[buf][8 * j + 4 * half]);
                }
                const int lo_[4] = {lo4.x, lo4.y, lo4.z, lo4.w}, hi_[4] = {hi4.x, hi4.y, hi4.z, hi4.w};
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const bool vis = (qpos[rb] >= lo_[i]) && (qpos[rb] <= hi_[i]);
                    const float x = vis ? s[rb][4 * j + i] * a.scale_log2e : -INFINITY;
                    sc[4 * j + i] = x;
                    mt = fmaxf(mt, x);
                }
            }
            mt = fmaxf(mt, __shfl_xor(mt, 32));  // the other 16 keys of this query
            const float mnew = fmaxf(m[rb], mt);
            const float msafe = mnew == -INFINITY ? 0.f : mnew;
            const float corr = __builtin_amdgcn_exp2f(m[rb] - msafe);
            float ps = 0.f;
            float p[16];
#pragma unroll
            for (int c = 0; c < 16; c++) p[c] = __builtin_amdgcn_exp2f(sc[c] - msafe);
#pragma unroll
            for (int c = 0; c < 8; c++) {
                pb[rb][c] = pf_pack(p[2 * c], p[2 * c + 1]);
                ps += __uint_as_float(pb[rb][c] << 16) + __uint_as_float(pb[rb][c] & 0xffff0000u);  // the rounded weights
            }
            l[rb] = l[rb] * corr + ps;
            if (__builtin_amdgcn_ballot_w64(mnew > m[rb]) != 0) {
#pragma unroll
                for (int db = 0; db < 4; db++)
#pragma unroll
                    for (int c = 0; c < 16; c++) o[rb][db][c] *= corr;
            }
            m[rb] = mnew;
        }
        // ---- O^T += V^T P^T : rows = d, columns = queries, contraction over the 32 keys ----
#pragma unroll
        for (int t2 = 0; t2 < 2; t2++) {
            pf_bf16x8_t pbv[2];
#pragma unroll
            for (int rb = 0; rb < 2; rb++) {
                const uint4 u4 = make_uint4(pb[rb][4 * t2], pb[rb][4 * t2 + 1], pb[rb][4 * t2 + 2], pb[rb][4 * t2 + 3]);
                pbv[rb] = __builtin_bit_cast(pf_bf16x8_t, u4);
            }
#pragma unroll
            for (int db = 0; db < 4; db++) {
                // the lane's 8 contraction slots are keys 16*t2 + 4*half + {0..3} and + 8 more
                const char *vp = &s_vt[buf][(db * 32 + qn) * kPfVStride + (16 * t2 + 4 * half) * 2];
                const uint2 v0 = *reinterpret_cast<const uint2 *>(vp);
                const uint2 v1 = *reinterpret_cast<const uint2 *>(vp + 16);
                const uint4 u4 = make_uint4(v0.x, v0.y, v1.x, v1.y);
                const pf_bf16x8_t va = __builtin_bit_cast(pf_bf16x8_t, u4);
                o[0][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pbv[0], o[0][db], 0, 0, 0);
                o[1][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pbv[1], o[1][db], 0, 0, 0);
            }
        }
        if (t + 1 < n_tiles) stage(buf ^ 1);
        __syncthreads();
    }

    // ---- normalise and write: register c = 4j+i of o[rb][db] is d = 32*db + 8j + 4*half + i ----
#pragma unroll
    for (int rb = 0; rb < 2; rb++) {
        const int i = qt * kPfQ + rb * 32 + qn;
        const float lt = l[rb] + __shfl_xor(l[rb], 32);
        if (i < T) {
            const float inv = 1.0f / lt;
            float *op = a.out + ((size_t)(base + i) * pv.Hq + (size_t)h * G + wave) * kPfD;
#pragma unroll
            for (int db = 0; db < 4; db++)
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    const float4 w4 = make_float4(o[rb][db][4 * j] * inv, o[rb][db][4 * j + 1] * inv,
                                                  o[rb][db][4 * j + 2] * inv, o[rb][db][4 * j + 3] * inv);
                    *reinterpret_cast<float4 *>(op + 32 * db + 8 * j + 4 * half) = w4;
                }
        }
    }
}

size_t attend_prefill_ws_bytes(const View &pv, int n_seqs, int64_t total_q) {
    (void)pv; (void)n_seqs; (void)total_q;
    return 256;  // the kernel keeps everything in registers and LDS
}

hipError_t launch_attend_prefill(const View &pv, const CallSeqs &cs, int layer, const void *q,
                                 const void *k, const void *v, const float *g, float tau,
                                 float scale, float *out, void *ws, hipStream_t st) {
    (void)ws;
    if (pv.dtype != WGKV_BF16 || pv.d != kPfD || pv.G != 4) return hipErrorNotSupported;
    PrefillAttnArgs a;
    a.layer = layer;
    a.tau = tau;
    a.scale_log2e = scale * 1.4426950408889634f;
    a.q = (const char *)q;
    a.k = (const char *)k;
    a.v = (const char *)v;
    a.g = g;
    a.out = out;
    int max_t = 0;
    for (int b = 0; b < cs.n; b++) max_t = max(max_t, cs.ntok[b]);
    if (max_t == 0) return hipSuccess;
    dim3 grid((max_t + kPfQ - 1) / kPfQ, pv.Hkv, cs.n);
    hipLaunchKernelGGL(attend_prefill_kernel, grid, dim3(256), 0, st, pv, cs, a);
    return hipGetLastError();
}

}  // namespace wgkv
