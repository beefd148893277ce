// Ragged, per-head paged GQA decode attention for gfx950 (wave64), bandwidth-bound.
//
// One query token per sequence.  A unit is one (sequence, kv head): its keys are
// the global cache [0, G_h) followed by the valid ring slots [0, min(t, W)); the
// G query heads of the group all read the same K/V rows (Sec. 4.3 last sentence,
// Sec. 2.1 equation; head-to-batch folding of App. A).  The cached tokens of all
// units, cut into 16-token tiles, form one long list that is split EVENLY over the
// waves of the launch -- a wave's share may start in the middle of one unit and end
// in the middle of another -- and every (wave, unit) overlap leaves a partial
// (m, l, acc); the wave that finishes a unit last folds the partials of that unit
// (the split-then-reduce balancing of App. E "Decode phase", taken down to tile
// granularity, without a second launch and without any wave waiting for another).
//
// Data path: each lane loads 16 bytes of a K row and of a V row straight into
// registers; 64 lanes x 16 B = 1 KiB per load instruction, fully coalesced.  A wave
// keeps several tiles in flight in separate register sets that are refilled in
// place as soon as they have been consumed, so that few waves per SIMD are enough
// to cover the HBM latency and no wave depends on the issue priority of another.
// A 16-lane (256-byte row) group owns one token per row, so a wave holds 64/LPT
// independent online-softmax streams that are only combined when a unit ends.
#include <type_traits>

#include <hip/hip_ext.h>

#include "wgkv_dev.h"

namespace wgkv {

constexpr int kTile = 16;        // tokens per tile
constexpr int kAttnThreads = 256;
constexpr int kAttnWaves = 4;
constexpr int kStagesFast = 4;   // tiles in flight per wave on the fast path
// A wave that begins a unit in the middle of its share drains its loads, publishes a partial and
// waits for the new unit's lengths, query rows and page ids; measured, the launch is shortest when
// that is priced at 10 to 16 tiles.
// The split charges it to the unit, as tiles in front of the first real one that nobody reads.
constexpr int kUnitStartTiles = 12;
// Blocks go to the XCDs round-robin, and in every launch measured the odd XCD of a pair streams
// slower than the even one, by 4-5 % on some machines and by about twice that on others: the
// waves of an odd block get a number of thousandths fewer tiles, those of the even block before
// it as many more (AttendArgs::skew_permille; 50 unless the pool was tuned on its machine, see
// wgkv_tune_decode_attention).
struct AttendArgs {
    int layer;
    int n_seqs;
    int min_tpw;              // at least this many tiles per wave
    int skew_permille;        // share of the odd blocks' tiles that goes to the even blocks instead
    float scale_log2e;        // scale * log2(e)
    const char *q;            // [n_seqs][Hq][d]
    float *out;               // [n_seqs][Hq][d]
    float *part_ml;           // [(waves + n_units)][G][2]
    float *part_acc;          // [(waves + n_units)][G][d]
    uint32_t part_ml_bytes, part_acc_bytes;
    int32_t *counters;        // [n_units] zero between calls: waves done per unit
    // optional page selection: only these pages of each head's global cache are read
    const int32_t *sel_pages; // [n_units][sel_stride] ascending indices into the head's global table, or NULL
    const int32_t *sel_count; // [n_units]
    int sel_stride;
    int32_t sid[kMaxCallSeqs];
};

// Tokens a unit reads from its global cache: all gl of them, or those of the selected pages (every
// page is full except possibly the last one of the cache, which then is the last one selected).
__device__ __forceinline__ int global_tokens(const View &pv, const AttendArgs &a, int u, int gl) {
    if (!a.sel_pages) return gl;
    const int n_pages = (gl + pv.P - 1) >> pv.logP;
    const int cnt = min(min(max(a.sel_count[u], 0), a.sel_stride), n_pages);
    if (cnt == 0) return 0;
    const int last = a.sel_pages[(size_t)u * a.sel_stride + cnt - 1];
    return (cnt - 1) * pv.P + (last >= n_pages - 1 ? gl - (n_pages - 1) * pv.P : pv.P);
}

__device__ __forceinline__ int ceil_tiles(int n) { return (n + kTile - 1) / kTile; }

// tiles of every unit -> exclusive prefix in s_ts[0..n_units]
__device__ __forceinline__ void build_tile_prefix(const View &pv, const AttendArgs &a, int n_units,
                                                  int *s_ts, int *s_tmp, int *s_gl, int *s_nl, int *s_um) {
    if (n_units <= 64) {  // one wave does it: a scan inside the wave, one barrier
        if (threadIdx.x < 64) {
            const int u = threadIdx.x;
            int tiles = 0;
            if (u < n_units) {
                const int b = u / pv.Hkv, h = u % pv.Hkv, sid = a.sid[b];
                const int t = pv.seq_len[sid * pv.L + a.layer];
                const int um = unit_meta(pv, sid, a.layer, h);
                const int gl_all = pv.global_len[um];
                const int gl = global_tokens(pv, a, u, gl_all);
                s_um[u] = um;
                s_gl[u] = gl_all;
                s_nl[u] = min(t, pv.W);
                tiles = ceil_tiles(gl) + ceil_tiles(min(t, pv.W));
                if (tiles > 0) tiles += kUnitStartTiles;
            }
            const int inc = wave_incl_scan(tiles, u);
            if (u < n_units) s_ts[u] = inc - tiles;
            if (u == 63) s_ts[n_units] = inc;
        }
        __syncthreads();
        return;
    }
    int carry = 0;
    for (int u0 = 0; u0 < n_units; u0 += kAttnThreads) {
        const int u = u0 + threadIdx.x;
        int tiles = 0;
        if (u < n_units) {
            const int b = u / pv.Hkv, h = u % pv.Hkv, sid = a.sid[b];
            const int t = pv.seq_len[sid * pv.L + a.layer];
            const int um = unit_meta(pv, sid, a.layer, h);
            const int gl_all = pv.global_len[um];
            const int gl = global_tokens(pv, a, u, gl_all);
            s_um[u] = um;
            s_gl[u] = gl_all;
            s_nl[u] = min(t, pv.W);
            tiles = ceil_tiles(gl) + ceil_tiles(min(t, pv.W));
            if (tiles > 0) tiles += kUnitStartTiles;
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
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {  // round to nearest even
    bf16x2_t t = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, t);
}
__device__ __forceinline__ float bf16_lo(uint32_t x) { return __uint_as_float(x << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t x) { return __uint_as_float(x & 0xffff0000u); }

// Partials cross compute units (and their L2 slices) inside one launch: they are
// written and read with device-coherent accesses, so no cache-wide flush is needed.
// Buffer accesses carry the same cache policy as a device-scope atomic access (sc1) at up to
// 16 bytes per lane, and an access outside the buffer reads zero or is dropped.
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
constexpr int kCoherent = 16;  // cache-policy operand of the buffer builtins: sc1
__device__ __forceinline__ __amdgpu_buffer_rsrc_t part_rsrc(float *p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(p, 0, (int)bytes, 0x00020000);  // raw buffer, 32-bit data format
}

template <int DT, int D, int G>
__global__ __launch_bounds__(kAttnThreads) void attend_decode_kernel(View pv, AttendArgs a) {
    constexpr int ES = Elem<DT>::es;
    constexpr int EPL = 16 / ES;      // elements per lane per row
    constexpr int LPT = D / EPL;      // lanes per token row
    constexpr int TPW = 64 / LPT;     // token rows per wave load
    constexpr int RPT = kTile / TPW;  // wave loads per tile (K and V each)
    constexpr int ROWB = D * ES;      // bytes of a K or V row
    static_assert(LPT == 8 || LPT == 16 || LPT == 32, "row must be 128, 256 or 512 bytes");
    // 256-byte rows with four query heads per kv head (every workload shape of the
    // paper's two models): the 16 scores of a tile are spread over the 16 lanes of a
    // row group, one per lane, so that max, exp and sum run once instead of 16 times.
    // In that mode m[0] and l[0] belong to head sub%4; the other entries are unused.
    constexpr bool FAST = (LPT == 16 && G == 4);
    constexpr int S = FAST ? kStagesFast : 1;  // register sets = tiles in flight

    __shared__ int s_ts[kMaxCallUnits + 1];
    __shared__ int s_gl[kMaxCallUnits];  // entries in the unit's global cache
    __shared__ int s_nl[kMaxCallUnits];  // tokens in its ring
    __shared__ int s_um[kMaxCallUnits];  // its index into the per-unit metadata
    __shared__ int s_tmp[20];
    __shared__ float s_p[kAttnWaves][64];          // fp32 weights of a tile (fp32 pool)
    __shared__ uint32_t s_pk[kAttnWaves][4][2][4]; // bf16 weight pairs of a tile: [row group][row pair][head]

    const int n_units = a.n_seqs * pv.Hkv;
    build_tile_prefix(pv, a, n_units, s_ts, s_tmp, s_gl, s_nl, s_um);
    const int total = s_ts[n_units];
    // units with nothing cached: the output is defined as zero (block b looks at units b, b + grid, ...:
    // one comparison for most blocks, nothing for the rest)
    for (int uu = blockIdx.x; uu < n_units; uu += gridDim.x)
        if (s_ts[uu + 1] == s_ts[uu]) {
            float *o = a.out + (size_t)uu * G * D;
            for (int i = threadIdx.x; i < G * D; i += kAttnThreads) o[i] = 0.f;
        }
    // From here on every wave works alone: no block-wide barrier below this line.
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane / LPT, sub = lane % LPT;
    const int n_waves = (int)gridDim.x * kAttnWaves;
    const int tpw = max(a.min_tpw, (total + n_waves - 1) / n_waves);
    const int wid = (int)blockIdx.x * kAttnWaves + wave;
    // shares: a pair of blocks (even, odd) covers 2 * kAttnWaves * tpw tiles, te per wave of the
    // even block and to per wave of the odd one
    const int skew = (gridDim.x % 2 == 0) ? tpw * a.skew_permille / 1000 : 0;
    const int te = tpw + skew, to = tpw - skew;
    constexpr int PW = 2 * kAttnWaves;
    auto wave_of = [&](int x) {  // the wave whose share holds tile x
        const int pr = x / (PW * tpw), r = x % (PW * tpw);
        return pr * PW + (r < kAttnWaves * te ? r / te : kAttnWaves + (r - kAttnWaves * te) / to);
    };
    const int widx = wid % PW;
    const int T0 = (wid / PW) * (PW * tpw) + (widx < kAttnWaves ? widx * te : kAttnWaves * te + (widx - kAttnWaves) * to);
    const int T1 = min(total, T0 + (widx < kAttnWaves ? te : to));
    if (T0 >= T1) return;

    // first unit of the share: the u with s_ts[u] <= T0 < s_ts[u+1]
    int u;
    if (n_units <= 64) {  // one comparison per lane: the units whose first tile is at or before T0
        const bool le = lane < n_units && s_ts[lane] <= T0;  // true for lane 0: s_ts[0] = 0
        u = __builtin_popcountll(__builtin_amdgcn_ballot_w64(le)) - 1;
    } else {
        int lo = 0, hi = n_units - 1;
        while (lo < hi) {
            int mid = (lo + hi + 1) >> 1;
            if (s_ts[mid] <= T0) lo = mid; else hi = mid - 1;
        }
        u = lo;
    }
    int cur = T0;
    while (cur < T1) {
        while (s_ts[u + 1] <= cur) u++;  // also skips units without tiles
        const int u_begin = s_ts[u] + kUnitStartTiles, u_end = min(s_ts[u + 1], T1);  // the unit's real tiles
        if (cur < u_begin) {
            cur = u_begin;
            if (cur >= T1) break;  // the share ends inside the allowance: the next wave begins the unit
        }
        // unit u = (sequence b of the call, kv head h): its query rows are rows u*G .. u*G+G-1 of q and out
        const int um = s_um[u];
        const int gl_all = s_gl[u];
        const int gl = global_tokens(pv, a, u, gl_all);
        const int nloc = s_nl[u];
        const int n_gt = ceil_tiles(gl);

        // this lane's slice of the G query rows
        uint32_t qreg[G][4];
        {
            const char *qp = a.q + ((size_t)u * G * D) * ES + sub * 16;
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
            // one piece: at most 64 tiles [k0, k0+n) of one region (global or local) of unit u
            const int kk = cur - u_begin;
            const bool is_glob = kk < n_gt;
            const int k0 = is_glob ? kk : kk - n_gt;
            const int region_tiles = is_glob ? n_gt : ceil_tiles(nloc);
            const int count = is_glob ? gl : nloc;
            const int n = min(min(region_tiles - k0, 64), u_end - cur);
            const int32_t *pt = is_glob ? pv.global_pt + (size_t)um * pv.maxgp
                                        : pv.local_pt + (size_t)um * pv.nlp;
            // A tile inside one page (P >= 16) needs one page id for the whole wave:
            // lane i keeps the page id of tile k0+i and the base address goes through
            // scalar registers.  In a partly filled last tile the rows beyond the last token
            // read the last valid row again and get weight zero: nothing that is not a cached
            // row of this head is ever read (a recycled page keeps whatever its last owner
            // left in it, which need not be finite).  With pages smaller than a tile every
            // tile is handled one at a time with a page lookup per row.
            // page id of the vp-th page of the region as this call reads it (with a selection: the
            // vp-th selected page; an index outside the table is clamped, never followed)
            const int32_t *sel = (is_glob && a.sel_pages) ? a.sel_pages + (size_t)u * a.sel_stride : nullptr;
            const int last_page = max(((gl_all + pv.P - 1) >> pv.logP) - 1, 0);
            auto page_at = [&](int vp) { return pt[sel ? min(max(sel[vp], 0), last_page) : vp]; };
            const bool page_per_tile = pv.logP >= 4;
            const int n_fast = page_per_tile ? n : 0;
            int ptreg = 0;

            // Row addresses of tile j (clamped to the last tile of the piece: a tile asked
            // for beyond the end is re-read and never used).  No memory access.
            auto tile_rows = [&](int j, const char *(&rowp)[RPT]) {
                j = min(j, n_fast - 1);
                const int k = k0 + j;
                const int page = __builtin_amdgcn_readlane(ptreg, j);
                const char *base = page_ptr(pv, page) + (size_t)((k * kTile) & (pv.P - 1)) * ROWB;
                const int last_row = count - 1 - k * kTile;  // wave-uniform; >= kTile - 1 except in the last tile
#pragma unroll
                for (int r = 0; r < RPT; r++)
                    rowp[r] = base + ((uint32_t)min(grp + r * TPW, last_row) * ROWB + (uint32_t)(sub * 16));
            };
            // Row addresses of any tile, one page lookup per row.
            auto tile_rows_any = [&](int j, const char *(&rowp)[RPT]) {
                const int k = k0 + j;
#pragma unroll
                for (int r = 0; r < RPT; r++) {
                    int tok = k * kTile + r * TPW + grp;
                    tok = min(tok, count - 1);  // rows past the end re-read a valid row and get weight 0
                    const int page = page_at(tok >> pv.logP);
                    rowp[r] = page_ptr(pv, page) + (size_t)(tok & (pv.P - 1)) * ROWB + sub * 16;
                }
            };

            uint4 kb[S][RPT], vb[S][RPT];

            // One tile out of register set ST; the set is refilled with tile j+S.
            auto process = [&](auto st_tag, auto refill_tag, int j) {
                constexpr int ST = decltype(st_tag)::value;
                constexpr bool REFILL = decltype(refill_tag)::value;
                const int k = k0 + j;
                const char *rowp[RPT];
                if constexpr (REFILL) tile_rows(j + S, rowp);
                if constexpr (FAST) {
                    // ---- 16 partial dot products per lane: x[r*4+g]; a K row register is
                    //      refilled as soon as it has been used ----
                    float x[16];
#pragma unroll
                    for (int r = 0; r < 4; r++) {
                        const uint32_t kw[4] = {kb[ST][r].x, kb[ST][r].y, kb[ST][r].z, kb[ST][r].w};
#pragma unroll
                        for (int g = 0; g < 4; g++) {
                            float d = 0.f;
                            if (DT == WGKV_BF16) {
#pragma unroll
                                for (int e = 0; e < 4; e++) d = dot2_bf16(kw[e], qreg[g][e], d);
                            } else {
#pragma unroll
                                for (int e = 0; e < 4; e++) d = fmaf(__uint_as_float(kw[e]), __uint_as_float(qreg[g][e]), d);
                            }
                            x[r * 4 + g] = d;
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        if constexpr (REFILL) kb[ST][r] = load_once16(rowp[r]);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    // ---- reduce-scatter over the 16 lanes of the row group: lane `sub`
                    //      ends up with the full dot product x[sub], i.e. row sub/4, head sub%4 ----
                    float y8[8], y4[4], y2[2];
#pragma unroll
                    for (int i = 0; i < 8; i++) {
                        const float lo_ = x[i] + dpp_f<kDppRor8>(x[i]);
                        const float hi_ = x[i + 8] + dpp_f<kDppRor8>(x[i + 8]);
                        y8[i] = (sub & 8) ? hi_ : lo_;
                    }
#pragma unroll
                    for (int i = 0; i < 4; i++) {
                        const float lo_ = y8[i] + dpp_f<kDppShl4>(y8[i]);
                        const float hi_ = y8[i + 4] + dpp_f<kDppShr4>(y8[i + 4]);
                        y4[i] = (sub & 4) ? hi_ : lo_;
                    }
#pragma unroll
                    for (int i = 0; i < 2; i++) {
                        const float lo_ = y4[i] + dpp_f<kDppXor2>(y4[i]);
                        const float hi_ = y4[i + 2] + dpp_f<kDppXor2>(y4[i + 2]);
                        y2[i] = (sub & 2) ? hi_ : lo_;
                    }
                    float sc;
                    {
                        const float lo_ = y2[0] + dpp_f<kDppXor1>(y2[0]);
                        const float hi_ = y2[1] + dpp_f<kDppXor1>(y2[1]);
                        sc = (sub & 1) ? hi_ : lo_;
                    }
                    const int tok_l = k * kTile + (sub >> 2) * TPW + grp;
                    sc = tok_l < count ? sc * a.scale_log2e : -INFINITY;
                    // ---- online softmax on one (row, head) per lane; lanes sub, sub^4, sub^8,
                    //      sub^12 hold the four rows of the same head ----
                    float mt = fmaxf(sc, dpp_f<kDppRor8>(sc));
                    mt = fmaxf(mt, dpp_f<kDppRor4>(mt));
                    const float mnew = fmaxf(m[0], mt);
                    const float msafe = mnew == -INFINITY ? 0.f : mnew;
                    const float corr = __builtin_amdgcn_exp2f(m[0] - msafe);
                    float pl = __builtin_amdgcn_exp2f(sc - msafe);
                    uint32_t pb = 0;
                    if constexpr (DT == WGKV_BF16) {
                        // the weights enter the weighted sum as bf16 pairs (rows 2i, 2i+1);
                        // the denominator sums the same rounded values
                        pb = pack_bf16(pl, dpp_f<kDppShl4>(pl));
                        pl = bf16_lo(pb);
                    }
                    float ps = pl + dpp_f<kDppRor8>(pl);
                    ps += dpp_f<kDppRor4>(ps);
                    l[0] = l[0] * corr + ps;
                    if (__builtin_amdgcn_ballot_w64(mnew > m[0]) != 0) {  // rare once the maxima settle
                        const float c0 = dpp_f<0x00>(corr), c1 = dpp_f<0x55>(corr);
                        const float c2 = dpp_f<0xAA>(corr), c3 = dpp_f<0xFF>(corr);
#pragma unroll
                        for (int e = 0; e < EPL; e++) {
                            acc[0][e] *= c0; acc[1][e] *= c1; acc[2][e] *= c2; acc[3][e] *= c3;
                        }
                    }
                    m[0] = mnew;
                    // ---- weights back to the row layout through the wave's LDS strip ----
                    if constexpr (DT == WGKV_BF16) {
                        if ((sub & 4) == 0) s_pk[wave][grp][sub >> 3][sub & 3] = pb;
                        __builtin_amdgcn_wave_barrier();
                        const uint4 pk0 = *reinterpret_cast<const uint4 *>(&s_pk[wave][grp][0][0]);
                        const uint4 pk1 = *reinterpret_cast<const uint4 *>(&s_pk[wave][grp][1][0]);
                        const uint32_t pk[2][4] = {{pk0.x, pk0.y, pk0.z, pk0.w}, {pk1.x, pk1.y, pk1.z, pk1.w}};
#pragma unroll
                        for (int i = 0; i < 2; i++) {
                            const uint32_t va[4] = {vb[ST][2 * i].x, vb[ST][2 * i].y, vb[ST][2 * i].z, vb[ST][2 * i].w};
                            const uint32_t vc[4] = {vb[ST][2 * i + 1].x, vb[ST][2 * i + 1].y, vb[ST][2 * i + 1].z,
                                                    vb[ST][2 * i + 1].w};
#pragma unroll
                            for (int e = 0; e < 4; e++) {
                                const uint32_t lo2 = __builtin_amdgcn_perm(vc[e], va[e], 0x05040100u);
                                const uint32_t hi2 = __builtin_amdgcn_perm(vc[e], va[e], 0x07060302u);
#pragma unroll
                                for (int g = 0; g < 4; g++) {
                                    acc[g][2 * e] = dot2_bf16(lo2, pk[i][g], acc[g][2 * e]);
                                    acc[g][2 * e + 1] = dot2_bf16(hi2, pk[i][g], acc[g][2 * e + 1]);
                                }
                            }
                            __builtin_amdgcn_sched_barrier(0);
                            if constexpr (REFILL) {
                                vb[ST][2 * i] = load_once16(rowp[2 * i] + pv.v_off);
                                vb[ST][2 * i + 1] = load_once16(rowp[2 * i + 1] + pv.v_off);
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        __builtin_amdgcn_wave_barrier();
                    } else {
                        s_p[wave][lane] = pl;
                        __builtin_amdgcn_wave_barrier();
#pragma unroll
                        for (int r = 0; r < 4; r++) {
                            const float4 pr = *reinterpret_cast<const float4 *>(&s_p[wave][grp * 16 + r * 4]);
                            const float pg[4] = {pr.x, pr.y, pr.z, pr.w};
                            const uint32_t vw[4] = {vb[ST][r].x, vb[ST][r].y, vb[ST][r].z, vb[ST][r].w};
#pragma unroll
                            for (int e = 0; e < 4; e++)
#pragma unroll
                                for (int g = 0; g < 4; g++) acc[g][e] = fmaf(pg[g], __uint_as_float(vw[e]), acc[g][e]);
                            __builtin_amdgcn_sched_barrier(0);
                            if constexpr (REFILL) vb[ST][r] = load_once16(rowp[r] + pv.v_off);
                            __builtin_amdgcn_sched_barrier(0);
                        }
                        __builtin_amdgcn_wave_barrier();
                    }
                } else {
                    // ---- scores of the tile, every lane of a row group gets all of them ----
                    float s[RPT][G];
#pragma unroll
                    for (int r = 0; r < RPT; r++) {
                        const uint32_t kw[4] = {kb[ST][r].x, kb[ST][r].y, kb[ST][r].z, kb[ST][r].w};
                        const int tok = k * kTile + r * TPW + grp;
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
                            s[r][g] = tok < count ? d * a.scale_log2e : -INFINITY;
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);  // the K registers are free from here on
                    if constexpr (REFILL) {
#pragma unroll
                        for (int r = 0; r < RPT; r++) kb[ST][r] = load_once16(rowp[r]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    // ---- online softmax per query head, one rescale per tile ----
                    float p[RPT][G];
#pragma unroll
                    for (int g = 0; g < G; g++) {
                        float mt = s[0][g];
#pragma unroll
                        for (int r = 1; r < RPT; r++) mt = fmaxf(mt, s[r][g]);
                        const float mnew = fmaxf(m[g], mt);
                        const float msafe = mnew == -INFINITY ? 0.f : mnew;
                        const float corr = __builtin_amdgcn_exp2f(m[g] - msafe);
                        m[g] = mnew;
                        float ps = 0.f;
#pragma unroll
                        for (int r = 0; r < RPT; r++) {
                            p[r][g] = __builtin_amdgcn_exp2f(s[r][g] - msafe);
                            ps += p[r][g];
                        }
                        l[g] = l[g] * corr + ps;
#pragma unroll
                        for (int e = 0; e < EPL; e++) acc[g][e] *= corr;
                    }
#pragma unroll
                    for (int r = 0; r < RPT; r++) {
                        const uint32_t vw[4] = {vb[ST][r].x, vb[ST][r].y, vb[ST][r].z, vb[ST][r].w};
                        if (DT == WGKV_BF16) {
#pragma unroll
                            for (int e = 0; e < 4; e++) {
                                const float vlo = bf16_lo(vw[e]), vhi = bf16_hi(vw[e]);
#pragma unroll
                                for (int g = 0; g < G; g++) {
                                    acc[g][2 * e] = fmaf(p[r][g], vlo, acc[g][2 * e]);
                                    acc[g][2 * e + 1] = fmaf(p[r][g], vhi, acc[g][2 * e + 1]);
                                }
                            }
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; e++)
#pragma unroll
                                for (int g = 0; g < G; g++) acc[g][e] = fmaf(p[r][g], __uint_as_float(vw[e]), acc[g][e]);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);  // the V registers are free from here on
                    if constexpr (REFILL) {
#pragma unroll
                        for (int r = 0; r < RPT; r++) vb[ST][r] = load_once16(rowp[r] + pv.v_off);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            };

            if (n_fast > 0) {
                ptreg = page_at(((k0 + min(lane, n_fast - 1)) * kTile) >> pv.logP);
                // prologue: fill every register set
#pragma unroll
                for (int st = 0; st < S; st++) {
                    const char *rowp[RPT];
                    tile_rows(st, rowp);
#pragma unroll
                    for (int r = 0; r < RPT; r++) kb[st][r] = load_once16(rowp[r]);
#pragma unroll
                    for (int r = 0; r < RPT; r++) vb[st][r] = load_once16(rowp[r] + pv.v_off);
                }
                // Main loop: S tiles per trip, straight-line, so that every wait is for exactly
                // the load that is needed and the younger ones stay in flight.  It runs while every
                // refill is a real tile of the piece.
                using std::integral_constant;
                constexpr std::true_type kRefill{};
                constexpr std::false_type kNoRefill{};
                static_assert(S == 1 || S == 4, "the loops below are written out for 1 or 4 register sets");
                int j = 0;
                if constexpr (S == 4) {
                    for (; j + 2 * S <= n_fast; j += S) {
                        process(integral_constant<int, 0>{}, kRefill, j);
                        process(integral_constant<int, 1>{}, kRefill, j + 1);
                        process(integral_constant<int, 2>{}, kRefill, j + 2);
                        process(integral_constant<int, 3>{}, kRefill, j + 3);
                    }
                    // the last full trip: only the first n_fast - j - S sets still have a tile to fetch
                    // (a set without one is left alone: asking again for the last tile would be traffic
                    // for nothing)
                    if (j + S <= n_fast) {
                        const int more = n_fast - j - S;
                        if (more > 0) process(integral_constant<int, 0>{}, kRefill, j);
                        else process(integral_constant<int, 0>{}, kNoRefill, j);
                        if (more > 1) process(integral_constant<int, 1>{}, kRefill, j + 1);
                        else process(integral_constant<int, 1>{}, kNoRefill, j + 1);
                        if (more > 2) process(integral_constant<int, 2>{}, kRefill, j + 2);
                        else process(integral_constant<int, 2>{}, kNoRefill, j + 2);
                        process(integral_constant<int, 3>{}, kNoRefill, j + 3);
                        j += S;
                    }
                    // the last n_fast % S tiles are already in their register sets
                    if (j < n_fast) process(integral_constant<int, 0>{}, kNoRefill, j);
                    if (j + 1 < n_fast) process(integral_constant<int, 1>{}, kNoRefill, j + 1);
                    if (j + 2 < n_fast) process(integral_constant<int, 2>{}, kNoRefill, j + 2);
                } else {
                    for (; j + 1 < n_fast; j++) process(integral_constant<int, 0>{}, kRefill, j);
                    if (j < n_fast) process(integral_constant<int, 0>{}, kNoRefill, j);
                }
            }
            // whatever is left of the piece, one tile at a time through register set 0
            for (int j = n_fast; j < n; j++) {
                const char *rowp[RPT];
                tile_rows_any(j, rowp);
#pragma unroll
                for (int r = 0; r < RPT; r++) kb[0][r] = load_once16(rowp[r]);
#pragma unroll
                for (int r = 0; r < RPT; r++) vb[0][r] = load_once16(rowp[r] + pv.v_off);
                process(std::integral_constant<int, 0>{}, std::false_type{}, j);
            }
            cur += n;
        }

        // ---- the unit (or the share) ends: fold the wave's row groups into one state ----
        if constexpr (FAST) {  // back to one (m, l) per head in every lane
            const float m1 = m[0], l1 = l[0];
            m[0] = dpp_f<0x00>(m1); m[1] = dpp_f<0x55>(m1); m[2] = dpp_f<0xAA>(m1); m[3] = dpp_f<0xFF>(m1);
            l[0] = dpp_f<0x00>(l1); l[1] = dpp_f<0x55>(l1); l[2] = dpp_f<0xAA>(l1); l[3] = dpp_f<0xFF>(l1);
        }
        auto merge_groups = [&](auto off_tag) __attribute__((always_inline)) {
            constexpr int OFF = decltype(off_tag)::value;
#pragma unroll
            for (int g = 0; g < G; g++) {
                const float mo = lane_xor<OFF>(m[g], lane), lo_ = lane_xor<OFF>(l[g], lane);
                const float mn = fmaxf(m[g], mo);
                const float ms = mn == -INFINITY ? 0.f : mn;
                const float ca = __builtin_amdgcn_exp2f(m[g] - ms), cb = __builtin_amdgcn_exp2f(mo - ms);
                l[g] = l[g] * ca + lo_ * cb;
#pragma unroll
                for (int e = 0; e < EPL; e++) acc[g][e] = acc[g][e] * ca + lane_xor<OFF>(acc[g][e], lane) * cb;
                m[g] = mn;
            }
        };
        if constexpr (LPT <= 8) merge_groups(std::integral_constant<int, 8>{});
        if constexpr (LPT <= 16) merge_groups(std::integral_constant<int, 16>{});
        merge_groups(std::integral_constant<int, 32>{});
        // waves whose share overlaps this unit
        const int w_first = wave_of(s_ts[u] + kUnitStartTiles), w_last = wave_of(s_ts[u + 1] - 1);
        float *o = a.out + (size_t)u * G * D;
        if (w_first == w_last) {  // the unit lies inside this wave's share
            if (lane < LPT) {
#pragma unroll
                for (int g = 0; g < G; g++) {
                    const float inv = 1.0f / l[g];
#pragma unroll
                    for (int e = 0; e < EPL; e++) o[g * D + sub * EPL + e] = acc[g][e] * inv;
                }
            }
        } else {
            // Partials: per (slot, head) the d values as [16-byte chunk of a lane][lane of the row
            // group][4], so that one store or load of a row group covers contiguous memory.  Every
            // row group holds the folded state; group grp handles heads grp, grp + NG, ...
            constexpr int NG = TPW, GT = (G + NG - 1) / NG, NJ = EPL / 4;
            const __amdgpu_buffer_rsrc_t r_acc = part_rsrc(a.part_acc, a.part_acc_bytes);
            const __amdgpu_buffer_rsrc_t r_ml = part_rsrc(a.part_ml, a.part_ml_bytes);
            const uint32_t slot = (uint32_t)(wid + u);
#pragma unroll
            for (int t = 0; t < GT; t++) {
                // the state of head grp + NG * t, picked without indexing registers by a run-time value
                float v[EPL], vm = m[NG * t], vl = l[NG * t];
#pragma unroll
                for (int e = 0; e < EPL; e++) v[e] = acc[NG * t][e];
#pragma unroll
                for (int gg = 1; gg < NG; gg++) {
                    constexpr int last = G - 1;
                    const int gs = NG * t + gg < G ? NG * t + gg : last;
                    if (NG * t + gg < G && grp == gg) {
                        vm = m[gs];
                        vl = l[gs];
#pragma unroll
                        for (int e = 0; e < EPL; e++) v[e] = acc[gs][e];
                    }
                }
                const int g = grp + NG * t;
                if (g < G) {
                    const uint32_t rec = slot * G + g;
#pragma unroll
                    for (int j = 0; j < NJ; j++) {
                        const u32x4 pk = {__float_as_uint(v[4 * j]), __float_as_uint(v[4 * j + 1]),
                                          __float_as_uint(v[4 * j + 2]), __float_as_uint(v[4 * j + 3])};
                        __builtin_amdgcn_raw_buffer_store_b128(pk, r_acc, rec * (D * 4) + (j * LPT + sub) * 16, 0, kCoherent);
                    }
                    if (sub == 0) {
                        const u32x2 pk = {__float_as_uint(vm), __float_as_uint(vl)};
                        __builtin_amdgcn_raw_buffer_store_b64(pk, r_ml, rec * 8, 0, kCoherent);
                    }
                }
            }
            // The folding wave usually sits on another compute unit, often on another XCD, so the
            // partial must be complete at device scope before the count moves.  The stores above
            // carry the device-scope policy (written through, not left dirty in this XCD's L2), and
            // on this architecture vmcnt counts stores until they are acknowledged at their scope:
            // the wave waits for all of them here, then issues the increment.  (An agent-scope
            // release fence says the same in the language's terms, but it also writes back the
            // whole L2 in front of the wait, and its acquire twin invalidates it: measured 117.5
            // instead of 86.6 us per launch on the 128K workload.)
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            int prev = 0;
            if (lane == 0) prev = __hip_atomic_fetch_add(&a.counters[u], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            prev = __builtin_amdgcn_readfirstlane(prev);
            if (prev == w_last - w_first) {  // every other wave of this unit is done: fold
                // The loads below are issued after the count has come back (the branch depends on
                // it) and bypass the caches that are not coherent at device scope; the compiler
                // must not move them in front of the atomic either.
                asm volatile("" ::: "memory");
                float Mx[GT], Ls[GT], A[GT][EPL];
#pragma unroll
                for (int t = 0; t < GT; t++) {
                    Mx[t] = -INFINITY;
                    Ls[t] = 0.f;
#pragma unroll
                    for (int e = 0; e < EPL; e++) A[t][e] = 0.f;
                }
                // the partials sit in device-coherent memory, one round trip away: ask for
                // several of them, 16 bytes a lane and load, before folding any
                constexpr int R = GT * (EPL + 2);  // registers one partial takes
                constexpr int BUD = FAST ? 160 : 80;  // registers the batch may take without costing the main loop waves
                constexpr int MB = BUD / R > 16 ? 16 : (BUD / R < 2 ? 2 : BUD / R);
                static_assert(MB * GT * (NJ + 1) < 64, "more loads in flight than the wave can count");
                for (int w0 = w_first; w0 <= w_last; w0 += MB) {
                    u32x2 mlv[MB][GT];
                    u32x4 av[MB][GT][NJ];
#pragma unroll
                    for (int i = 0; i < MB; i++) {
                        const uint32_t sl = (uint32_t)(min(w0 + i, w_last) + u);
#pragma unroll
                        for (int t = 0; t < GT; t++) {
                            const uint32_t rec = sl * G + min(grp + NG * t, G - 1);
                            mlv[i][t] = __builtin_amdgcn_raw_buffer_load_b64(r_ml, rec * 8, 0, kCoherent);
#pragma unroll
                            for (int j = 0; j < NJ; j++)
                                av[i][t][j] = __builtin_amdgcn_raw_buffer_load_b128(r_acc, rec * (D * 4) + (j * LPT + sub) * 16, 0, kCoherent);
                        }
                    }
#pragma unroll
                    for (int i = 0; i < MB; i++) {
                        if (w0 + i <= w_last) {
#pragma unroll
                            for (int t = 0; t < GT; t++) {
                                const float mi = __uint_as_float(mlv[i][t].x), li = __uint_as_float(mlv[i][t].y);
                                const float mn = fmaxf(Mx[t], mi);
                                const float ms = mn == -INFINITY ? 0.f : mn;
                                const float ca = __builtin_amdgcn_exp2f(Mx[t] - ms), cb = __builtin_amdgcn_exp2f(mi - ms);
                                Ls[t] = Ls[t] * ca + li * cb;
#pragma unroll
                                for (int j = 0; j < NJ; j++) {
                                    A[t][4 * j] = A[t][4 * j] * ca + __uint_as_float(av[i][t][j].x) * cb;
                                    A[t][4 * j + 1] = A[t][4 * j + 1] * ca + __uint_as_float(av[i][t][j].y) * cb;
                                    A[t][4 * j + 2] = A[t][4 * j + 2] * ca + __uint_as_float(av[i][t][j].z) * cb;
                                    A[t][4 * j + 3] = A[t][4 * j + 3] * ca + __uint_as_float(av[i][t][j].w) * cb;
                                }
                                Mx[t] = mn;
                            }
                        }
                    }
                }
#pragma unroll
                for (int t = 0; t < GT; t++) {
                    const int g = grp + NG * t;
                    if (g < G) {
                        const float inv = 1.0f / Ls[t];
#pragma unroll
                        for (int e = 0; e < EPL; e++) o[g * D + sub * EPL + e] = A[t][e] * inv;
                    }
                }
                if (lane == 0) __hip_atomic_store(&a.counters[u], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    }
}

// Blocks of one instantiation that fit on a compute unit at the same time.  The
// launch uses exactly (compute units x that many) blocks: with an even split of the
// tiles a second, partly filled round of blocks would double the run time.
template <int DT, int D, int GG>
static int resident_blocks_per_cu() {
    static int cached = 0;
    if (cached == 0) {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, attend_decode_kernel<DT, D, GG>, kAttnThreads, 0) != hipSuccess || n < 1)
            n = 1;
        cached = n;
    }
    return cached;
}

template <int DT, int D>
static hipError_t launch_g(const View &pv, const AttendArgs &a, int n_cu, int grid_max, hipStream_t st,
                           hipEvent_t ev0, hipEvent_t ev1) {
    int grid = 0;
    switch (pv.G) {
#define WGKV_CASE(GG)                                                                              \
    case GG:                                                                                       \
        grid = n_cu * resident_blocks_per_cu<DT, D, GG>();                                         \
        if (grid > grid_max) grid = grid_max;                                                      \
        if (ev0 && ev1)  /* the events take the begin and end time stamps of this dispatch itself */ \
            hipExtLaunchKernelGGL((attend_decode_kernel<DT, D, GG>), dim3(grid), dim3(kAttnThreads), 0, st, ev0, ev1, 0, pv, a); \
        else                                                                                       \
            hipLaunchKernelGGL((attend_decode_kernel<DT, D, GG>), dim3(grid), dim3(kAttnThreads), 0, st, pv, a); \
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

// workspace bytes for a decode attend launched with at most grid_max blocks
size_t attend_decode_ws_bytes(const View &pv, int n_seqs, int grid_max) {
    const size_t n_units = (size_t)n_seqs * pv.Hkv, slots = (size_t)grid_max * kAttnWaves + n_units;
    size_t b = slots * pv.G * 2 * sizeof(float);
    b = (b + 255) & ~(size_t)255;
    b += slots * pv.G * pv.d * sizeof(float);
    return b;
}

// ---- scratch for callers that bring no workspace ----
// One array per GPU, part of the loaded code object: it exists from the moment the library is
// loaded on a device until the process ends.  In host code the array's name is only a handle
// for hipGetSymbolAddress; the address that kernels and copies use is the one that call returns,
// looked up once per device while that device is current.
static __device__ __align__(256) unsigned char scratch[WGKV_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each device, NULL = not looked up yet

hipError_t static_scratch_init() {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (g_scratch_ptr[dev]) return hipSuccess;
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
    return hipSuccess;
}

// The current device's scratch array, or NULL when static_scratch_init has not run on it.
void *static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    return g_scratch_ptr[dev];
}

// Fills the occupancy cache of the pool's instantiation, so that no later launch asks the runtime.
template <int DT, int D>
static void warm_g(int G) {
    switch (G) {
        case 1: resident_blocks_per_cu<DT, D, 1>(); break;
        case 2: resident_blocks_per_cu<DT, D, 2>(); break;
        case 4: resident_blocks_per_cu<DT, D, 4>(); break;
        case 8: resident_blocks_per_cu<DT, D, 8>(); break;
        default: break;
    }
}
void attend_decode_warm(const View &pv) {
    if (pv.dtype == WGKV_BF16 && pv.d == 128) warm_g<WGKV_BF16, 128>(pv.G);
    if (pv.dtype == WGKV_BF16 && pv.d == 64) warm_g<WGKV_BF16, 64>(pv.G);
    if (pv.dtype == WGKV_F32 && pv.d == 128) warm_g<WGKV_F32, 128>(pv.G);
    if (pv.dtype == WGKV_F32 && pv.d == 64) warm_g<WGKV_F32, 64>(pv.G);
}

hipError_t launch_attend_decode(const View &pv, int layer, int n_seqs, const int32_t *sids,
                                const void *q, float scale, float *out, void *ws, int32_t *counters,
                                int n_cu, int grid_max, int min_tpw, hipStream_t st, hipEvent_t ev0,
                                hipEvent_t ev1, const int32_t *sel_pages, const int32_t *sel_count,
                                int sel_stride, int skew_permille) {
    AttendArgs a;
    a.skew_permille = skew_permille;
    a.sel_pages = sel_pages;
    a.sel_count = sel_count;
    a.sel_stride = sel_stride;
    a.layer = layer;
    a.n_seqs = n_seqs;
    a.min_tpw = min_tpw;
    a.scale_log2e = scale * 1.4426950408889634f;
    a.q = (const char *)q;
    a.out = out;
    a.counters = counters;
    // the partial slots are laid out for the largest grid any instantiation may use
    const size_t n_units = (size_t)n_seqs * pv.Hkv, slots = (size_t)grid_max * kAttnWaves + n_units;
    char *w = (char *)ws;
    a.part_ml = (float *)w;
    size_t off = (slots * pv.G * 2 * sizeof(float) + 255) & ~(size_t)255;
    a.part_acc = (float *)(w + off);
    const size_t acc_bytes = slots * pv.G * pv.d * sizeof(float);
    if (acc_bytes > 0x7fffffffu) return hipErrorInvalidValue;  // 32-bit offsets into the partials
    a.part_ml_bytes = (uint32_t)(slots * pv.G * 2 * sizeof(float));
    a.part_acc_bytes = (uint32_t)acc_bytes;
    for (int i = 0; i < n_seqs; i++) a.sid[i] = sids[i];
    if (pv.dtype == WGKV_BF16 && pv.d == 128) return launch_g<WGKV_BF16, 128>(pv, a, n_cu, grid_max, st, ev0, ev1);
    if (pv.dtype == WGKV_BF16 && pv.d == 64) return launch_g<WGKV_BF16, 64>(pv, a, n_cu, grid_max, st, ev0, ev1);
    if (pv.dtype == WGKV_F32 && pv.d == 128) return launch_g<WGKV_F32, 128>(pv, a, n_cu, grid_max, st, ev0, ev1);
    if (pv.dtype == WGKV_F32 && pv.d == 64) return launch_g<WGKV_F32, 64>(pv, a, n_cu, grid_max, st, ev0, ev1);
    return hipErrorInvalidValue;
}

}  // namespace wgkv
