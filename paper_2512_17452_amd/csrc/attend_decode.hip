// Ragged, per-head paged GQA decode attention for gfx950 (wave64), bandwidth-bound.
//
// One query token per sequence.  A unit is one (sequence, kv head): its keys are
// the global cache [0, G_h) followed by the valid ring slots [0, min(t, W)); the
// G query heads of the group all read the same K/V rows (Sec. 4.3 last sentence,
// Sec. 2.1 equation; head-to-batch folding of App. A).  The cached tokens of all
// units, cut into 16-token tiles, form one long list that is split EVENLY over the
// blocks of the launch -- a block's share may start in the middle of one unit and
// end in the middle of another -- and every (block, unit) overlap leaves a partial
// (m, l, acc) that a second kernel merges (the split-then-reduce balancing of
// App. E "Decode phase", taken down to tile granularity).
//
// Data path: each lane loads 16 bytes of a K row and of a V row straight into
// registers; 64 lanes x 16 B = 1 KiB per load instruction, fully coalesced, next
// tile in flight while the current one is reduced.  A 16-lane (256-byte row) group
// owns one token per row, so a wave holds 64/LPT independent online-softmax
// streams that are only combined when a unit ends.
#include "wgkv_dev.h"

namespace wgkv {

constexpr int kTile = 16;        // tokens per tile
constexpr int kAttnThreads = 256;
constexpr int kAttnWaves = 4;
constexpr int kPtStage = 1056;   // page ids staged in LDS per piece

struct AttendArgs {
    int layer;
    int n_seqs;
    int min_tpb;              // at least this many tiles per block
    float scale_log2e;        // scale * log2(e)
    const char *q;            // [n_seqs][Hq][d]
    float *out;               // [n_seqs][Hq][d]
    float *part_ml;           // [(grid + n_units)][G][2]
    float *part_acc;          // [(grid + n_units)][G][d]
    int32_t *tile_start;      // [n_units + 1] written by block 0 for the merge kernel
    int32_t sid[kMaxCallSeqs];
};

__device__ __forceinline__ int ceil_tiles(int n) { return (n + kTile - 1) / kTile; }

// tiles of every unit -> exclusive prefix in s_ts[0..n_units]
__device__ __forceinline__ void build_tile_prefix(const View &pv, const AttendArgs &a, int n_units,
                                                  int *s_ts, int *s_tmp) {
    int carry = 0;
    for (int u0 = 0; u0 < n_units; u0 += kAttnThreads) {
        const int u = u0 + threadIdx.x;
        int tiles = 0;
        if (u < n_units) {
            const int b = u / pv.Hkv, h = u % pv.Hkv, sid = a.sid[b];
            const int t = pv.seq_len[sid * pv.L + a.layer];
            const int gl = pv.global_len[unit_meta(pv, sid, a.layer, h)];
            tiles = ceil_tiles(gl) + ceil_tiles(min(t, pv.W));
        }
        int total;
        const int ex = block_excl_scan(tiles, s_tmp, &total);
        if (u < n_units) s_ts[u] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) s_ts[n_units] = carry;
    __syncthreads();
}

template <int DT> struct Elem;
template <> struct Elem<WGKV_F32> { static constexpr int es = 4; };
template <> struct Elem<WGKV_BF16> { static constexpr int es = 2; };

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                           __builtin_bit_cast(bf16x2_t, b), c, false);
}
__device__ __forceinline__ float bf16_lo(uint32_t x) { return __uint_as_float(x << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t x) { return __uint_as_float(x & 0xffff0000u); }

template <int DT, int D, int G>
__global__ __launch_bounds__(kAttnThreads) void attend_decode_kernel(View pv, AttendArgs a) {
    constexpr int ES = Elem<DT>::es;
    constexpr int EPL = 16 / ES;      // elements per lane per row
    constexpr int LPT = D / EPL;      // lanes per token row
    constexpr int TPW = 64 / LPT;     // token rows per wave load
    constexpr int RPT = kTile / TPW;  // wave loads per tile (K and V each)
    static_assert(LPT == 8 || LPT == 16 || LPT == 32, "row must be 128, 256 or 512 bytes");

    __shared__ int s_ts[kMaxCallUnits + 1];
    __shared__ int s_tmp[20];
    __shared__ int s_pt[kPtStage];
    __shared__ float s_m[kAttnWaves][G], s_l[kAttnWaves][G];
    __shared__ float s_acc[kAttnWaves][G][D];

    const int n_units = a.n_seqs * pv.Hkv;
    build_tile_prefix(pv, a, n_units, s_ts, s_tmp);
    const int total = s_ts[n_units];
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i <= n_units; i += kAttnThreads) a.tile_start[i] = s_ts[i];
    const int tpb = max(a.min_tpb, (total + (int)gridDim.x - 1) / (int)gridDim.x);
    const int T0 = blockIdx.x * tpb;
    const int T1 = min(total, T0 + tpb);
    if (T0 >= T1) return;  // block-uniform

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane / LPT, sub = lane % LPT;

    // first unit of the share: largest u with s_ts[u] <= T0 and s_ts[u+1] > T0
    int u;
    {
        int lo = 0, hi = n_units - 1;
        while (lo < hi) {
            int mid = (lo + hi + 1) >> 1;
            if (s_ts[mid] <= T0) lo = mid; else hi = mid - 1;
        }
        u = lo;
        while (s_ts[u + 1] <= T0) u++;  // skip units without tiles
    }

    int cur = T0;
    while (cur < T1) {
        while (s_ts[u + 1] <= cur) u++;
        const int b = u / pv.Hkv, h = u % pv.Hkv, sid = a.sid[b];
        const int um = unit_meta(pv, sid, a.layer, h);
        const int gl = pv.global_len[um];
        const int nloc = min(pv.seq_len[sid * pv.L + a.layer], pv.W);
        const int n_gt = ceil_tiles(gl);
        const int u_begin = s_ts[u], u_end = min(s_ts[u + 1], T1);

        // this lane's slice of the G query rows
        uint32_t qreg[G][4];
        {
            const char *qp = a.q + ((size_t)(b * pv.Hq + h * G) * D) * ES + sub * 16;
#pragma unroll
            for (int g = 0; g < G; g++) {
                const uint4 t4 = *reinterpret_cast<const uint4 *>(qp + (size_t)g * D * ES);
                qreg[g][0] = t4.x; qreg[g][1] = t4.y; qreg[g][2] = t4.z; qreg[g][3] = t4.w;
            }
        }
        float m[G], l[G], acc[G][EPL];
#pragma unroll
        for (int g = 0; g < G; g++) {
            m[g] = -INFINITY;
            l[g] = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; e++) acc[g][e] = 0.f;
        }

        while (cur < u_end) {
            // one piece: tiles [k0, k1) of one region (global or local) of unit u
            const int kk = cur - u_begin;
            const bool is_glob = kk < n_gt;
            const int k0 = is_glob ? kk : kk - n_gt;
            const int region_tiles = is_glob ? n_gt : ceil_tiles(nloc);
            const int count = is_glob ? gl : nloc;
            const int piece_cap = pv.logP >= 4 ? 1024 : (64 << pv.logP);
            const int k1 = min(min(region_tiles, k0 + piece_cap), k0 + (u_end - cur));
            const int32_t *pt = is_glob ? pv.global_pt + (size_t)um * pv.maxgp
                                        : pv.local_pt + (size_t)um * pv.nlp;
            const int page0 = (k0 * kTile) >> pv.logP;
            const int page1 = (min(k1 * kTile, count) - 1) >> pv.logP;
            __syncthreads();  // previous piece is done with s_pt
            for (int i = threadIdx.x; i <= page1 - page0; i += kAttnThreads) s_pt[i] = pt[page0 + i];
            __syncthreads();

            uint4 kb[RPT], vb[RPT], kn[RPT], vn[RPT];
            auto load_tile = [&](int k, uint4 *kd, uint4 *vd) {
#pragma unroll
                for (int r = 0; r < RPT; r++) {
                    int tok = k * kTile + r * TPW + grp;
                    tok = min(tok, count - 1);
                    const int page = s_pt[(tok >> pv.logP) - page0];
                    const char *p = page_ptr(pv, page) + (size_t)(tok & (pv.P - 1)) * pv.row_bytes + sub * 16;
                    kd[r] = *reinterpret_cast<const uint4 *>(p);
                    vd[r] = *reinterpret_cast<const uint4 *>(p + pv.v_off);
                }
            };
            int k = k0 + wave;
            if (k < k1) load_tile(k, kb, vb);
            while (k < k1) {
                const int kn_i = k + kAttnWaves;
                if (kn_i < k1) load_tile(kn_i, kn, vn);
                // ---- scores of the tile: s[r][g] ----
                float s[RPT][G];
#pragma unroll
                for (int r = 0; r < RPT; r++) {
                    const uint32_t kw[4] = {kb[r].x, kb[r].y, kb[r].z, kb[r].w};
#pragma unroll
                    for (int g = 0; g < G; g++) {
                        float d = 0.f;
                        if (DT == WGKV_BF16) {
#pragma unroll
                            for (int e = 0; e < 4; e++) d = dot2_bf16(kw[e], qreg[g][e], d);
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; e++) d = fmaf(__uint_as_float(kw[e]), __uint_as_float(qreg[g][e]), d);
                        }
                        d = group_sum<LPT>(d);
                        const int tok = k * kTile + r * TPW + grp;
                        s[r][g] = tok < count ? d * a.scale_log2e : -INFINITY;
                    }
                }
                // ---- online softmax per query head, one rescale per tile ----
#pragma unroll
                for (int g = 0; g < G; g++) {
                    float mt = s[0][g];
#pragma unroll
                    for (int r = 1; r < RPT; r++) mt = fmaxf(mt, s[r][g]);
                    const float mnew = fmaxf(m[g], mt);
                    const float msafe = mnew == -INFINITY ? 0.f : mnew;
                    const float corr = __builtin_amdgcn_exp2f(m[g] - msafe);
                    m[g] = mnew;
                    float p[RPT], ps = 0.f;
#pragma unroll
                    for (int r = 0; r < RPT; r++) {
                        p[r] = __builtin_amdgcn_exp2f(s[r][g] - msafe);
                        ps += p[r];
                    }
                    l[g] = l[g] * corr + ps;
#pragma unroll
                    for (int e = 0; e < EPL; e++) acc[g][e] *= corr;
#pragma unroll
                    for (int r = 0; r < RPT; r++) {
                        const uint32_t vw[4] = {vb[r].x, vb[r].y, vb[r].z, vb[r].w};
                        if (DT == WGKV_BF16) {
#pragma unroll
                            for (int e = 0; e < 4; e++) {
                                acc[g][2 * e] = fmaf(p[r], bf16_lo(vw[e]), acc[g][2 * e]);
                                acc[g][2 * e + 1] = fmaf(p[r], bf16_hi(vw[e]), acc[g][2 * e + 1]);
                            }
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; e++) acc[g][e] = fmaf(p[r], __uint_as_float(vw[e]), acc[g][e]);
                        }
                    }
                }
#pragma unroll
                for (int r = 0; r < RPT; r++) { kb[r] = kn[r]; vb[r] = vn[r]; }
                k = kn_i;
            }
            cur += k1 - k0;
        }

        // ---- unit (or share) ends: combine the streams of the block, write one partial ----
#pragma unroll
        for (int off = LPT; off < 64; off <<= 1) {
#pragma unroll
            for (int g = 0; g < G; g++) {
                const float mo = __shfl_xor(m[g], off), lo_ = __shfl_xor(l[g], off);
                const float mn = fmaxf(m[g], mo);
                const float ms = mn == -INFINITY ? 0.f : mn;
                const float ca = __builtin_amdgcn_exp2f(m[g] - ms), cb = __builtin_amdgcn_exp2f(mo - ms);
                l[g] = l[g] * ca + lo_ * cb;
#pragma unroll
                for (int e = 0; e < EPL; e++) acc[g][e] = acc[g][e] * ca + __shfl_xor(acc[g][e], off) * cb;
                m[g] = mn;
            }
        }
        __syncthreads();  // s_acc free again
        if (lane < LPT) {
#pragma unroll
            for (int g = 0; g < G; g++) {
                if (sub == 0) { s_m[wave][g] = m[g]; s_l[wave][g] = l[g]; }
#pragma unroll
                for (int e = 0; e < EPL; e++) s_acc[wave][g][sub * EPL + e] = acc[g][e];
            }
        }
        __syncthreads();
        const size_t slot = (size_t)blockIdx.x + u;
        for (int i = threadIdx.x; i < G * D; i += kAttnThreads) {
            const int g = i / D, e = i % D;
            float mm = s_m[0][g];
#pragma unroll
            for (int w = 1; w < kAttnWaves; w++) mm = fmaxf(mm, s_m[w][g]);
            const float ms = mm == -INFINITY ? 0.f : mm;
            float ll = 0.f, aa = 0.f;
#pragma unroll
            for (int w = 0; w < kAttnWaves; w++) {
                const float c = __builtin_amdgcn_exp2f(s_m[w][g] - ms);
                ll += s_l[w][g] * c;
                aa += s_acc[w][g][e] * c;
            }
            a.part_acc[(slot * G + g) * D + e] = aa;
            if (e == 0) {
                a.part_ml[(slot * G + g) * 2] = mm;
                a.part_ml[(slot * G + g) * 2 + 1] = ll;
            }
        }
    }
}

// One block per unit: fold the partials of the blocks that overlapped it.
template <int D, int G>
__global__ __launch_bounds__(256) void attend_merge_kernel(View pv, AttendArgs a, int grid_main) {
    const int u = blockIdx.x;
    const int n_units = a.n_seqs * pv.Hkv;
    const int total = a.tile_start[n_units];
    const int ts0 = a.tile_start[u], ts1 = a.tile_start[u + 1];
    const int b = u / pv.Hkv, h = u % pv.Hkv;
    float *o = a.out + ((size_t)b * pv.Hq + (size_t)h * G) * D;
    if (ts1 <= ts0) {  // nothing cached for this unit
        for (int i = threadIdx.x; i < G * D; i += 256) o[i] = 0.f;
        return;
    }
    const int tpb = max(a.min_tpb, (total + grid_main - 1) / grid_main);
    const int b0 = ts0 / tpb, b1 = (ts1 - 1) / tpb;
    for (int i = threadIdx.x; i < G * D; i += 256) {
        const int g = i / D, e = i % D;
        float mm = -INFINITY;
        for (int bb = b0; bb <= b1; bb++) mm = fmaxf(mm, a.part_ml[((size_t)(bb + u) * G + g) * 2]);
        const float ms = mm == -INFINITY ? 0.f : mm;
        float ll = 0.f, aa = 0.f;
        for (int bb = b0; bb <= b1; bb++) {
            const size_t s = (size_t)(bb + u) * G + g;
            const float c = __builtin_amdgcn_exp2f(a.part_ml[s * 2] - ms);
            ll += a.part_ml[s * 2 + 1] * c;
            aa += a.part_acc[s * D + e] * c;
        }
        o[i] = aa / ll;
    }
}

template <int DT, int D>
static hipError_t launch_g(const View &pv, const AttendArgs &a, int grid, hipStream_t st,
                           hipEvent_t ev0, hipEvent_t ev1) {
    const int n_units = a.n_seqs * pv.Hkv;
    if (ev0) (void)hipEventRecord(ev0, st);
    switch (pv.G) {
#define WGKV_CASE(GG)                                                                              \
    case GG:                                                                                       \
        hipLaunchKernelGGL((attend_decode_kernel<DT, D, GG>), dim3(grid), dim3(kAttnThreads), 0, st, pv, a); \
        if (ev1) (void)hipEventRecord(ev1, st);                                                    \
        hipLaunchKernelGGL((attend_merge_kernel<D, GG>), dim3(n_units), dim3(256), 0, st, pv, a, grid);   \
        break;
        WGKV_CASE(1)
        WGKV_CASE(2)
        WGKV_CASE(4)
        WGKV_CASE(8)
#undef WGKV_CASE
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// workspace bytes for a decode attend with this grid
size_t attend_decode_ws_bytes(const View &pv, int n_seqs, int grid) {
    const size_t n_units = (size_t)n_seqs * pv.Hkv, slots = grid + n_units;
    size_t b = (n_units + 1) * sizeof(int32_t);
    b = (b + 255) & ~(size_t)255;
    b += slots * pv.G * 2 * sizeof(float);
    b = (b + 255) & ~(size_t)255;
    b += slots * pv.G * pv.d * sizeof(float);
    return b;
}

hipError_t launch_attend_decode(const View &pv, int layer, int n_seqs, const int32_t *sids,
                                const void *q, float scale, float *out, void *ws, int grid,
                                int min_tpb, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
    AttendArgs a;
    a.layer = layer;
    a.n_seqs = n_seqs;
    a.min_tpb = min_tpb;
    a.scale_log2e = scale * 1.4426950408889634f;
    a.q = (const char *)q;
    a.out = out;
    const size_t n_units = (size_t)n_seqs * pv.Hkv, slots = grid + n_units;
    char *w = (char *)ws;
    a.tile_start = (int32_t *)w;
    size_t off = ((n_units + 1) * sizeof(int32_t) + 255) & ~(size_t)255;
    a.part_ml = (float *)(w + off);
    off += slots * pv.G * 2 * sizeof(float);
    off = (off + 255) & ~(size_t)255;
    a.part_acc = (float *)(w + off);
    for (int i = 0; i < n_seqs; i++) a.sid[i] = sids[i];
    if (pv.dtype == WGKV_BF16 && pv.d == 128) return launch_g<WGKV_BF16, 128>(pv, a, grid, st, ev0, ev1);
    if (pv.dtype == WGKV_BF16 && pv.d == 64) return launch_g<WGKV_BF16, 64>(pv, a, grid, st, ev0, ev1);
    if (pv.dtype == WGKV_F32 && pv.d == 128) return launch_g<WGKV_F32, 128>(pv, a, grid, st, ev0, ev1);
    if (pv.dtype == WGKV_F32 && pv.d == 64) return launch_g<WGKV_F32, 64>(pv, a, grid, st, ev0, ev1);
    return hipErrorInvalidValue;
}

}  // namespace wgkv
