// Chunk attention under the vertical-slash mask (Sec. 4.2 "Vertical-slash sparse attention"; mask equation of
// Sec. 4.2 on the attention of Sec. 2.1) for the shapes the matrix-core kernel does not take: fp32 pools,
// head_dim 64, group sizes other than 4.  Plain vector arithmetic, fp32 accumulation, no LDS.
//
// One wave per (query position, query head).  Its keys are, in this order, the head's global cache (all visible:
// admitted and older than every window of the chunk), the ring (oldest position first) and the chunk up to the
// query itself; a ring or chunk key at position p is visible to the query at position i iff i - p < W or its
// score >= tau.  Per tile of 64 keys: lane j forms the whole dot product of key j with the query (the query sits
// in registers, every lane holds all of it), the wave takes the maximum and rescales (online softmax in the
// base-2 domain), then for every visible key the lanes, now spread over the head dimension, add p_j * v_j.
#include "wgkv_dev.h"

namespace wgkv {

struct PlainPrefillArgs {
    int layer;
    float tau, scale_log2e;
    int64_t total_q;        // queries of the call (all sequences)
    const char *q, *k, *v;  // chunk tensors of the pool's dtype
    const float *g;         // chunk scores
    float *out;
};

template <int DT> struct PlainElem;
template <> struct PlainElem<WGKV_BF16> {
    static constexpr int es = 2;
    // 16 bytes = 8 values
    static __device__ __forceinline__ void unpack(const uint4 &u, float (&f)[8]) {
        f[0] = __uint_as_float(u.x << 16); f[1] = __uint_as_float(u.x & 0xffff0000u);
        f[2] = __uint_as_float(u.y << 16); f[3] = __uint_as_float(u.y & 0xffff0000u);
        f[4] = __uint_as_float(u.z << 16); f[5] = __uint_as_float(u.z & 0xffff0000u);
        f[6] = __uint_as_float(u.w << 16); f[7] = __uint_as_float(u.w & 0xffff0000u);
    }
    static __device__ __forceinline__ float load1(const char *row, int e) {
        return __uint_as_float((uint32_t)*reinterpret_cast<const uint16_t *>(row + 2 * e) << 16);
    }
};
template <> struct PlainElem<WGKV_F32> {
    static constexpr int es = 4;
    static __device__ __forceinline__ float load1(const char *row, int e) {
        return *reinterpret_cast<const float *>(row + 4 * e);
    }
};

template <int DT, int D>
__global__ __launch_bounds__(256) void attend_prefill_plain_kernel(View pv, CallSeqs cs, PlainPrefillArgs a) {
    using E = PlainElem<DT>;
    constexpr int ROWB = D * E::es;
    constexpr int EPL = D / 64;  // output elements per lane
    const int lane = threadIdx.x & 63;
    const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);  // (query row of the call, query head)
    if (item >= a.total_q * pv.Hq) return;  // wave-uniform; the kernel has no barrier
    const int row_q = (int)(item / pv.Hq), qh = (int)(item % pv.Hq);
    const int h = qh / pv.G;
    int b = 0;
    while (b + 1 < cs.n && row_q >= cs.base[b + 1]) b++;  // sequences are packed in call order
    const int i = row_q - cs.base[b];
    const int t0 = cs.t0[b], base = cs.base[b];
    const int um = unit_meta(pv, cs.sid[b], a.layer, h);
    const int gl = pv.global_len[um];
    const int w_eff = min(pv.W, t0);              // ring entries that exist
    const int slot0 = t0 > pv.W ? t0 % pv.W : 0;  // ring slot of the oldest position
    const int qpos = t0 + i;
    const int n_keys = gl + w_eff + i + 1;

    // the query, all of it in every lane
    float qf[D];
    {
        const char *qp = a.q + ((size_t)row_q * pv.Hq + qh) * ROWB;
        if constexpr (DT == WGKV_BF16) {
#pragma unroll
            for (int c = 0; c < D / 8; c++) {
                float f[8];
                E::unpack(*reinterpret_cast<const uint4 *>(qp + 16 * c), f);
#pragma unroll
                for (int e = 0; e < 8; e++) qf[8 * c + e] = f[e];
            }
        } else {
#pragma unroll
            for (int c = 0; c < D / 4; c++) {
                const float4 f = *reinterpret_cast<const float4 *>(qp + 16 * c);
                qf[4 * c] = f.x; qf[4 * c + 1] = f.y; qf[4 * c + 2] = f.z; qf[4 * c + 3] = f.w;
            }
        }
    }
    float m = -INFINITY, l = 0.f, acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; e++) acc[e] = 0.f;

    for (int j0 = 0; j0 < n_keys; j0 += 64) {
        const int j = j0 + lane;
        // where key j lives and whether the query sees it
        const char *kp = a.k, *vp = a.v;  // lanes past the end read the first row of the chunk and drop it
        bool vis = false;
        if (j < gl) {
            const int pg = pv.global_pt[(size_t)um * pv.maxgp + (j >> pv.logP)];
            kp = page_ptr(pv, pg) + (size_t)(j & (pv.P - 1)) * ROWB;
            vp = kp + pv.v_off;
            vis = true;
        } else if (j < gl + w_eff) {
            const int idx = j - gl;
            int slot = slot0 + idx;
            slot = slot >= pv.W ? slot - pv.W : slot;
            const int pg = pv.local_pt[(size_t)um * pv.nlp + (slot >> pv.logP)];
            kp = page_ptr(pv, pg) + (size_t)(slot & (pv.P - 1)) * ROWB;
            vp = kp + pv.v_off;
            const int pos = t0 - w_eff + idx;
            vis = (qpos - pos < pv.W) || (pv.ring_g[(size_t)um * pv.W + slot] >= a.tau);
        } else if (j < n_keys) {
            const int idx = j - gl - w_eff;  // position t0 + idx <= qpos
            const size_t row = (size_t)(base + idx) * pv.Hkv + h;
            kp = a.k + row * ROWB;
            vp = a.v + row * ROWB;
            vis = (i - idx < pv.W) || (a.g[row] >= a.tau);
        }
        // score of this lane's key
        float s = 0.f;
        if constexpr (DT == WGKV_BF16) {
#pragma unroll
            for (int c = 0; c < D / 8; c++) {
                float f[8];
                E::unpack(*reinterpret_cast<const uint4 *>(kp + 16 * c), f);
#pragma unroll
                for (int e = 0; e < 8; e++) s = fmaf(qf[8 * c + e], f[e], s);
            }
        } else {
#pragma unroll
            for (int c = 0; c < D / 4; c++) {
                const float4 f = *reinterpret_cast<const float4 *>(kp + 16 * c);
                s = fmaf(qf[4 * c], f.x, s); s = fmaf(qf[4 * c + 1], f.y, s);
                s = fmaf(qf[4 * c + 2], f.z, s); s = fmaf(qf[4 * c + 3], f.w, s);
            }
        }
        s = vis ? s * a.scale_log2e : -INFINITY;
        float mt = s;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) mt = fmaxf(mt, __shfl_xor(mt, o));
        const float mnew = fmaxf(m, mt);
        if (mnew == -INFINITY) continue;  // nothing visible so far (wave-uniform)
        const float corr = __builtin_amdgcn_exp2f(m - mnew);  // 0 when m was -inf
        const float p = vis ? __builtin_amdgcn_exp2f(s - mnew) : 0.f;
        float ps = p;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) ps += __shfl_xor(ps, o);
        l = l * corr + ps;
        m = mnew;
#pragma unroll
        for (int e = 0; e < EPL; e++) acc[e] *= corr;
        // out += p_j v_j for the visible keys of the tile, the lanes over the head dimension
        uint64_t todo = __ballot(vis);
        const uint32_t vlo = (uint32_t)(uintptr_t)vp, vhi = (uint32_t)((uintptr_t)vp >> 32);
        while (todo) {
            const int jj = __builtin_ctzll(todo);
            todo &= todo - 1;
            const float pj = __shfl(p, jj);
            const char *vr = reinterpret_cast<const char *>(((uint64_t)(uint32_t)__shfl((int)vhi, jj) << 32) |
                                                            (uint32_t)__shfl((int)vlo, jj));
#pragma unroll
            for (int e = 0; e < EPL; e++) acc[e] = fmaf(pj, E::load1(vr, lane + 64 * e), acc[e]);
        }
    }
    float *op = a.out + ((size_t)row_q * pv.Hq + qh) * D;
    const float inv = 1.0f / l;
#pragma unroll
    for (int e = 0; e < EPL; e++) op[lane + 64 * e] = acc[e] * inv;
}

template <int DT, int D>
static hipError_t launch_plain_t(const View &pv, const CallSeqs &cs, const PlainPrefillArgs &a, hipStream_t st) {
    const int64_t items = a.total_q * pv.Hq;
    hipLaunchKernelGGL((attend_prefill_plain_kernel<DT, D>), dim3((unsigned)((items + 3) / 4)), dim3(256), 0, st, pv, cs, a);
    return hipGetLastError();
}

hipError_t launch_attend_prefill_plain(const View &pv, const CallSeqs &cs, int layer, const void *q, const void *k,
                                       const void *v, const float *g, float tau, float scale, float *out,
                                       hipStream_t st) {
    PlainPrefillArgs a;
    a.layer = layer;
    a.tau = tau;
    a.scale_log2e = scale * 1.4426950408889634f;
    a.total_q = 0;
    for (int b = 0; b < cs.n; b++) a.total_q += cs.ntok[b];
    a.q = (const char *)q;
    a.k = (const char *)k;
    a.v = (const char *)v;
    a.g = g;
    a.out = out;
    if (a.total_q == 0) return hipSuccess;
    if (a.total_q * pv.Hq >= ((int64_t)1 << 33)) return hipErrorInvalidValue;  // grid.x
    if (pv.dtype == WGKV_BF16 && pv.d == 128) return launch_plain_t<WGKV_BF16, 128>(pv, cs, a, st);
    if (pv.dtype == WGKV_BF16 && pv.d == 64) return launch_plain_t<WGKV_BF16, 64>(pv, cs, a, st);
    if (pv.dtype == WGKV_F32 && pv.d == 128) return launch_plain_t<WGKV_F32, 128>(pv, cs, a, st);
    if (pv.dtype == WGKV_F32 && pv.d == 64) return launch_plain_t<WGKV_F32, 64>(pv, cs, a, st);
    return hipErrorNotSupported;
}

}  // namespace wgkv
