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
// One block owns 64 chunk positions of one (sequence, kv head); its eight waves are
// (query head of the group) x (row block of 32 positions), so a K/V tile staged in LDS
// feeds all of them and two waves share each SIMD.
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

__global__ __launch_bounds__(512) void attend_prefill_kernel(View pv, CallSeqs cs, PrefillAttnArgs a) {
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
    // eight waves: wave -> (query head of the group, row block of 32 positions); two waves
    // share a SIMD, so one can run its softmax while the other keeps the matrix core busy
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int head = wave & 3, rb = wave >> 2;
    const int qn = lane & 31, half = lane >> 5;
    const int gl = pv.global_len[um];
    const int w_eff = min(pv.W, t0);              // ring entries that exist
    const int i_end = min(T, qt * kPfQ + kPfQ);   // chunk keys this block can see: [0, i_end)
    const int n_g = (gl + kPfKT - 1) / kPfKT, n_r = (w_eff + kPfKT - 1) / kPfKT;
    const int n_c = (i_end + kPfKT - 1) / kPfKT;
    const int n_tiles = n_g + n_r + n_c;

    // ---- Q^T operand: this lane's query, all 8 d-slices of 16 ----
    pf_bf16x8_t qv[8];
    const int qi = min(qt * kPfQ + rb * 32 + qn, T - 1);
    const int qpos = t0 + qi;
    {
        const char *qp = a.q + ((size_t)(base + qi) * pv.Hq + (size_t)h * G + head) * kPfD * 2;
#pragma unroll
        for (int ks = 0; ks < 8; ks++)
            qv[ks] = *reinterpret_cast<const pf_bf16x8_t *>(qp + (ks * 16 + half * 8) * 2);
    }
    pf_f32x16_t o[4];
    float m = -INFINITY, l = 0.f;
#pragma unroll
    for (int db = 0; db < 4; db++)
#pragma unroll
        for (int c = 0; c < 16; c++) o[db][c] = 0.f;

    // ---- staging of a key tile: thread -> (pair of keys 2j, 2j+1; 16-byte d chunk) ----
    // the two V rows of a pair are interleaved element-wise so that the transposed tile is
    // written with 32-bit stores
    const int ld_pair = threadIdx.x >> 5, ld_dc = threadIdx.x & 15, ld_sel = (threadIdx.x >> 4) & 1;
    // threads with ld_sel = 0 carry the K chunk of key 2j and the V chunks of both keys' low
    // half (d chunk ld_dc, elements 0..3); ld_sel = 1: K of key 2j+1 and elements 4..7
    const int ld_key = 2 * ld_pair + ld_sel;
    // two sets of staging registers: a tile is requested two iterations before it is multiplied
    struct StReg { uint4 kreg; uint2 vreg0, vreg1; int lo_reg, hi_reg; };
    StReg r0, r1;
    // Page ids live in registers, one per lane, so that the address of a key row never
    // waits for a page-table load: 64 consecutive entries of the global table (reloaded
    // every 64 pages) and the whole local table when it has at most 64 entries.
    int pt_base = 0;
    int ptreg = (lane < pv.maxgp) ? pv.global_pt[(size_t)um * pv.maxgp + lane] : 0;
    const bool lp_in_reg = pv.nlp <= 64;
    const int lpreg = (lp_in_reg && lane < pv.nlp) ? pv.local_pt[(size_t)um * pv.nlp + lane] : 0;
    const int slot0 = t0 > pv.W ? t0 % pv.W : 0;  // ring slot of the oldest position
    const int64_t v_delta_chunk = a.v - a.k;
    auto fetch = [&](int t, StReg &r) __attribute__((always_inline)) {
        const char *kp[2];
        int64_t v_delta;
        int lo[2] = {INT_MAX, INT_MAX}, hi[2] = {INT_MAX, INT_MAX};  // invisible unless shown otherwise
        if (t < n_g) {  // global cache: visible to every query
            if (((t * kPfKT + kPfKT - 1) >> pv.logP) >= pt_base + 64) {
                pt_base = (t * kPfKT) >> pv.logP;
                ptreg = (pt_base + lane < pv.maxgp) ? pv.global_pt[(size_t)um * pv.maxgp + pt_base + lane] : 0;
            }
#pragma unroll
            for (int e = 0; e < 2; e++) {
                const int idx = t * kPfKT + 2 * ld_pair + e, idc = min(idx, gl - 1);
                const int pg = __shfl(ptreg, (idc >> pv.logP) - pt_base);
                kp[e] = page_ptr(pv, pg) + (size_t)(idc & (pv.P - 1)) * (kPfD * 2);
                if (idx < gl) lo[e] = INT_MIN;
            }
            v_delta = pv.v_off;
        } else if (t < n_g + n_r) {  // ring, oldest position first
#pragma unroll
            for (int e = 0; e < 2; e++) {
                const int idx = (t - n_g) * kPfKT + 2 * ld_pair + e, idc = min(idx, w_eff - 1);
                int slot = slot0 + idc;
                slot = slot >= pv.W ? slot - pv.W : slot;
                const int pos = t0 - w_eff + idc;
                const int pg = lp_in_reg ? __shfl(lpreg, slot >> pv.logP)
                                         : pv.local_pt[(size_t)um * pv.nlp + (slot >> pv.logP)];
                kp[e] = page_ptr(pv, pg) + (size_t)(slot & (pv.P - 1)) * (kPfD * 2);
                if (idx < w_eff) {
                    lo[e] = pos;
                    hi[e] = (pv.ring_g[(size_t)um * pv.W + slot] >= a.tau) ? INT_MAX : pos + pv.W - 1;
                }
            }
            v_delta = pv.v_off;
        } else {  // this chunk
#pragma unroll
            for (int e = 0; e < 2; e++) {
                const int idx = (t - n_g - n_r) * kPfKT + 2 * ld_pair + e, idc = min(idx, T - 1);
                const size_t row = (size_t)(base + idc) * pv.Hkv + h;
                kp[e] = a.k + row * (kPfD * 2);
                if (idx < T) {
                    lo[e] = t0 + idx;
                    hi[e] = (a.g[row] >= a.tau) ? INT_MAX : t0 + idx + pv.W - 1;
                }
            }
            v_delta = v_delta_chunk;
        }
        r.kreg = *reinterpret_cast<const uint4 *>((ld_sel ? kp[1] : kp[0]) + ld_dc * 16);
        // V: the same 8-byte half chunk of both keys of the pair
        r.vreg0 = *reinterpret_cast<const uint2 *>(kp[0] + v_delta + ld_dc * 16 + ld_sel * 8);
        r.vreg1 = *reinterpret_cast<const uint2 *>(kp[1] + v_delta + ld_dc * 16 + ld_sel * 8);
        r.lo_reg = ld_sel ? lo[1] : lo[0];
        r.hi_reg = ld_sel ? hi[1] : hi[0];
    };
    // Full tiles of the global cache, pages of at least 4 tokens: the four keys a wave
    // stages share a page, so the page base is scalar and a lane only adds a fixed offset.
    const bool lean_ok = pv.P >= 4;
    const uint32_t lean_row = (uint32_t)((2 * ld_pair) & (pv.P - 1));
    const uint32_t lean_k_off = (lean_row + ld_sel) * (kPfD * 2) + ld_dc * 16;
    const uint32_t lean_v_off = lean_row * (kPfD * 2) + pv.v_off + ld_dc * 16 + ld_sel * 8;
    auto fetch_lean = [&](int t, StReg &r) __attribute__((always_inline)) {
        if (((t * kPfKT + kPfKT - 1) >> pv.logP) >= pt_base + 64) {
            pt_base = (t * kPfKT) >> pv.logP;
            ptreg = (pt_base + lane < pv.maxgp) ? pv.global_pt[(size_t)um * pv.maxgp + pt_base + lane] : 0;
        }
        const int pg = __builtin_amdgcn_readlane(ptreg, ((t * kPfKT + 4 * wave) >> pv.logP) - pt_base);
        const char *sb = page_ptr(pv, pg) + (size_t)((t * kPfKT) & (pv.P - 1)) * (kPfD * 2);
        r.kreg = *reinterpret_cast<const uint4 *>(sb + lean_k_off);
        r.vreg0 = *reinterpret_cast<const uint2 *>(sb + lean_v_off);
        r.vreg1 = *reinterpret_cast<const uint2 *>(sb + lean_v_off + kPfD * 2);
        r.lo_reg = INT_MIN;
        r.hi_reg = INT_MAX;
    };
    auto stage = [&](int buf, const StReg &r) __attribute__((always_inline)) {
        *reinterpret_cast<uint4 *>(&s_k[buf][ld_key * kPfKStride + ld_dc * 16]) = r.kreg;
        // transposed V: row d, columns (key 2j, key 2j+1) as one 32-bit word
        const uint32_t a0[2] = {r.vreg0.x, r.vreg0.y}, a1[2] = {r.vreg1.x, r.vreg1.y};
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const uint32_t x0 = (e & 1) ? (a0[e >> 1] >> 16) : (a0[e >> 1] & 0xffffu);
            const uint32_t x1 = (e & 1) ? (a1[e >> 1] & 0xffff0000u) : (a1[e >> 1] << 16);
            const int dd = ld_dc * 8 + ld_sel * 4 + e;
            *reinterpret_cast<uint32_t *>(&s_vt[buf][dd * kPfVStride + ld_pair * 4]) = x0 | x1;
        }
        if (ld_dc == 0) { s_lo[buf][ld_key] = r.lo_reg; s_hi[buf][ld_key] = r.hi_reg; }
    };

    const int n_plain = gl / kPfKT;  // full tiles of the global cache: no mask
    auto fetch_any = [&](int t, StReg &r) __attribute__((always_inline)) {
        if (lean_ok && t < n_plain) fetch_lean(t, r);
        else fetch(t, r);
    };
    fetch_any(0, r0);
    stage(0, r0);
    if (n_tiles > 1) fetch_any(1, r1);
    __syncthreads();

    // one iteration: tile t is multiplied, tile t+2 is requested into rf, tile t+1 goes from rs to LDS
    auto body = [&](int t, StReg &rf, const StReg &rs) __attribute__((always_inline)) {
        const int buf = t & 1;
        // LDS latency is the scarce thing here: the eight K fragments are requested at once,
        // the address arithmetic and global loads of the next tile run while they arrive,
        // and the V fragments are requested before the softmax that hides their latency.
        pf_bf16x8_t ka[8];
#pragma unroll
        for (int ks = 0; ks < 8; ks++)
            ka[ks] = *reinterpret_cast<const pf_bf16x8_t *>(&s_k[buf][qn * kPfKStride + (ks * 16 + half * 8) * 2]);
        __builtin_amdgcn_sched_barrier(0);
        if (t + 2 < n_tiles) fetch_any(t + 2, rf);  // in flight while this tile and the next are multiplied
        __builtin_amdgcn_sched_barrier(0);

        // ---- S^T = K Q^T : rows = keys of the tile, columns = this wave's queries ----
        pf_f32x16_t s;
#pragma unroll
        for (int c = 0; c < 16; c++) s[c] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ks++) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qv[ks], s, 0, 0, 0);
        // the lane's 8 contraction slots of V^T are keys 16*t2 + 4*half + {0..3} and + 8 more
        pf_bf16x8_t va[2][4];
#pragma unroll
        for (int t2 = 0; t2 < 2; t2++)
#pragma unroll
            for (int db = 0; db < 4; db++) {
                const char *vp = &s_vt[buf][(db * 32 + qn) * kPfVStride + (16 * t2 + 4 * half) * 2];
                const uint2 v0 = *reinterpret_cast<const uint2 *>(vp);
                const uint2 v1 = *reinterpret_cast<const uint2 *>(vp + 16);
                const uint4 u4 = make_uint4(v0.x, v0.y, v1.x, v1.y);
                va[t2][db] = __builtin_bit_cast(pf_bf16x8_t, u4);
            }
        __builtin_amdgcn_sched_barrier(0);
        // register c = 4j+i of a lane holds key 8j + 4*half + i of the tile
        const bool plain = t < n_plain;
        float sc[16];
        float mt = -INFINITY;
        if (plain) {
#pragma unroll
            for (int c = 0; c < 16; c++) {
                sc[c] = s[c] * a.scale_log2e;
                mt = fmaxf(mt, sc[c]);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const int4 lo4 = *reinterpret_cast<const int4 *>(&s_lo[buf][8 * j + 4 * half]);
                const int4 hi4 = *reinterpret_cast<const int4 *>(&s_hi[buf][8 * j + 4 * half]);
                const int lo_[4] = {lo4.x, lo4.y, lo4.z, lo4.w}, hi_[4] = {hi4.x, hi4.y, hi4.z, hi4.w};
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const bool vis = (qpos >= lo_[i]) && (qpos <= hi_[i]);
                    const float x = vis ? s[4 * j + i] * a.scale_log2e : -INFINITY;
                    sc[4 * j + i] = x;
                    mt = fmaxf(mt, x);
                }
            }
        }
        mt = fmaxf(mt, __shfl_xor(mt, 32));  // the other 16 keys of this query
        const float mnew = fmaxf(m, mt);
        const float msafe = mnew == -INFINITY ? 0.f : mnew;
        const float corr = __builtin_amdgcn_exp2f(m - msafe);
        uint32_t pb[8];
        float ps = 0.f;
        const pf_bf16x2_t ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
        for (int c = 0; c < 8; c++) {
            pb[c] = pf_pack(__builtin_amdgcn_exp2f(sc[2 * c] - msafe), __builtin_amdgcn_exp2f(sc[2 * c + 1] - msafe));
            // the denominator sums the rounded weights, the ones the second product uses
            ps = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(pf_bf16x2_t, pb[c]), ones, ps, false);
        }
        l = l * corr + ps;
        if (__builtin_amdgcn_ballot_w64(mnew > m) != 0) {
#pragma unroll
            for (int db = 0; db < 4; db++)
#pragma unroll
                for (int c = 0; c < 16; c++) o[db][c] *= corr;
        }
        m = mnew;
        // ---- O^T += V^T P^T : rows = d, columns = queries, contraction over the 32 keys ----
#pragma unroll
        for (int t2 = 0; t2 < 2; t2++) {
            const uint4 p4 = make_uint4(pb[4 * t2], pb[4 * t2 + 1], pb[4 * t2 + 2], pb[4 * t2 + 3]);
            const pf_bf16x8_t pbv = __builtin_bit_cast(pf_bf16x8_t, p4);
#pragma unroll
            for (int db = 0; db < 4; db++)
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[t2][db], pbv, o[db], 0, 0, 0);
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

    // ---- normalise and write: register c = 4j+i of o[db] is d = 32*db + 8j + 4*half + i ----
    {
        const int i = qt * kPfQ + rb * 32 + qn;
        const float lt = l + __shfl_xor(l, 32);
        if (i < T) {
            const float inv = 1.0f / lt;
            float *op = a.out + ((size_t)(base + i) * pv.Hq + (size_t)h * G + head) * kPfD;
#pragma unroll
            for (int db = 0; db < 4; db++)
#pragma unroll
                for (int j = 0; j < 4; j++) {
                    const float4 w4 = make_float4(o[db][4 * j] * inv, o[db][4 * j + 1] * inv,
                                                  o[db][4 * j + 2] * inv, o[db][4 * j + 3] * inv);
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
    hipLaunchKernelGGL(attend_prefill_kernel, grid, dim3(512), 0, st, pv, cs, a);
    return hipGetLastError();
}

}  // namespace wgkv
