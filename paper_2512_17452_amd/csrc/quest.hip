// Read-time page selection over the admitted cache (appendix "Synergy with KV Selection":
// Quest-style selection with key landmarks, the per-page minimum and maximum key vectors).
//
//  quest_update_kernel   landmarks of the pages that changed since the last update
//  quest_score_kernel    criticality of every page for a decode query:
//                        U_p = max over the group of sum_e max(q[e] lo_p[e], q[e] hi_p[e])
//  quest_select_kernel   the budget's worth of pages with the largest U, as ascending indices
//
// Landmarks are stored per physical page, in the pool's dtype (a minimum or maximum of stored
// values is a stored value): [n_pages][lo row, hi row][d], followed by one int32 per
// (sequence slot, layer, kv head): the number of entries the head's landmarks cover.
#include "wgkv_dev.h"

namespace wgkv {

struct QuestArgs {
    int layer;
    int reset;               // recompute every page of the given heads
    char *lm;                // landmarks [n_pages][2][d] of the pool dtype
    int32_t *lm_len;         // [S * L * Hkv]
    const char *q;           // [n_seqs][Hq][d]
    float *scores;           // [n_units][score_stride]
    long long score_stride;
    int budget_pages;
    int32_t *sel_pages;      // [n_units][budget_pages]
    int32_t *sel_count;      // [n_units]
};

template <int DT>
__device__ __forceinline__ float q_ld(const char *p, size_t i) {
    return DT == WGKV_F32 ? reinterpret_cast<const float *>(p)[i]
                          : __uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(p)[i] << 16);
}
template <int DT>
__device__ __forceinline__ void q_st(char *p, size_t i, float x) {
    if (DT == WGKV_F32) reinterpret_cast<float *>(p)[i] = x;
    else reinterpret_cast<uint16_t *>(p)[i] = (uint16_t)(__float_as_uint(x) >> 16);  // x is a bf16 value: exact
}

// Element-wise minimum / maximum of two 16-byte chunks of keys.
template <int DT>
__device__ __forceinline__ void q_minmax(uint4 &lo, uint4 &hi, const uint4 &x) {
    uint32_t *l = reinterpret_cast<uint32_t *>(&lo), *h = reinterpret_cast<uint32_t *>(&hi);
    const uint32_t *v = reinterpret_cast<const uint32_t *>(&x);
#pragma unroll
    for (int i = 0; i < 4; i++) {
        if (DT == WGKV_F32) {
            l[i] = __float_as_uint(fminf(__uint_as_float(l[i]), __uint_as_float(v[i])));
            h[i] = __float_as_uint(fmaxf(__uint_as_float(h[i]), __uint_as_float(v[i])));
        } else {  // two bf16 values per word; a minimum of bf16 values is one of them, so nothing is rounded
            const float l0 = fminf(__uint_as_float(l[i] << 16), __uint_as_float(v[i] << 16));
            const float l1 = fminf(__uint_as_float(l[i] & 0xffff0000u), __uint_as_float(v[i] & 0xffff0000u));
            const float h0 = fmaxf(__uint_as_float(h[i] << 16), __uint_as_float(v[i] << 16));
            const float h1 = fmaxf(__uint_as_float(h[i] & 0xffff0000u), __uint_as_float(v[i] & 0xffff0000u));
            l[i] = (__float_as_uint(l0) >> 16) | (__float_as_uint(l1) & 0xffff0000u);
            h[i] = (__float_as_uint(h0) >> 16) | (__float_as_uint(h1) & 0xffff0000u);
        }
    }
}

__device__ __forceinline__ uint4 q_shfl_xor(const uint4 &x, int m) {
    return make_uint4(__shfl_xor(x.x, m), __shfl_xor(x.y, m), __shfl_xor(x.z, m), __shfl_xor(x.w, m));
}

// One block per (sequence, kv head), one wave per page at a time.  A wave reads four rows of a page
// at once: 16 lanes per row, 16 bytes per lane (rows longer than 256 bytes take several turns).
template <int DT>
__global__ __launch_bounds__(256) void quest_update_kernel(View pv, CallSeqs cs, QuestArgs a) {
    const int u = blockIdx.x, b = u / pv.Hkv, h = u % pv.Hkv;
    const int um = unit_meta(pv, cs.sid[b], a.layer, h);
    const int N = pv.global_len[um];
    const int covered = a.reset ? 0 : min(a.lm_len[um], N);
    __syncthreads();  // everybody has read lm_len before it is rewritten below
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane & 15, rg = lane >> 4;
    const int p_end = (N + pv.P - 1) >> pv.logP, cpr = (int)(pv.row_bytes / 16);
    // the page that holds entry `covered` may have grown: start there
    for (int p = (covered >> pv.logP) + wave; p < p_end; p += 4) {
        const int page = pv.global_pt[(size_t)um * pv.maxgp + p];
        const int rows = min(pv.P, N - p * pv.P);
        const char *kp = page_ptr(pv, page);
        char *lo_row = a.lm + (size_t)page * 2 * pv.row_bytes, *hi_row = lo_row + pv.row_bytes;
        for (int c = sub; c < cpr; c += 16) {
            // row 0 exists; lanes whose first row is past the end start from it, which changes nothing
            uint4 lo = *reinterpret_cast<const uint4 *>(kp + (size_t)(rg < rows ? rg : 0) * pv.row_bytes + c * 16), hi = lo;
            for (int r = rg + 4; r < rows; r += 4)
                q_minmax<DT>(lo, hi, *reinterpret_cast<const uint4 *>(kp + (size_t)r * pv.row_bytes + c * 16));
            uint4 lo2 = q_shfl_xor(lo, 16), hi2 = q_shfl_xor(hi, 16);
            q_minmax<DT>(lo, hi, lo2);
            q_minmax<DT>(lo, hi, hi2);
            lo2 = q_shfl_xor(lo, 32);
            hi2 = q_shfl_xor(hi, 32);
            q_minmax<DT>(lo, hi, lo2);
            q_minmax<DT>(lo, hi, hi2);
            if (rg == 0) {
                *reinterpret_cast<uint4 *>(lo_row + c * 16) = lo;
                *reinterpret_cast<uint4 *>(hi_row + c * 16) = hi;
            }
        }
    }
    if (threadIdx.x == 0) a.lm_len[um] = N;
}

// Sixteen lanes per page, four pages per wave at a time and four such turns in flight; a lane reads 16 bytes
// of the minimum row and of the maximum row of a page, once for the whole group of query heads, whose queries sit
// in LDS as floats.  The launch is small (1/P of the keys), so its time is its chain of dependent loads: the page
// ids are asked for together with the head's length (entries past the last page hold -1 and the table row is
// maxgp wide, so the ids need no length to be read safely), which leaves two round trips, ids then landmarks;
// the grid is sized so that nearly every lane group has a single turn of four pages.
template <int DT, int G>
__global__ __launch_bounds__(256) void quest_score_kernel(View pv, CallSeqs cs, QuestArgs a) {
    extern __shared__ float s_q[];  // [G][d]
    constexpr int EPC = DT == WGKV_F32 ? 4 : 8;  // elements per 16-byte chunk
    constexpr int PF = 4;
    const int u = blockIdx.y, b = u / pv.Hkv, h = u % pv.Hkv;
    const int um = unit_meta(pv, cs.sid[b], a.layer, h);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane & 15, slot = lane >> 4, cpr = (int)(pv.row_bytes / 16);
    const int32_t *pt = pv.global_pt + (size_t)um * pv.maxgp;
    int pidx[PF], page[PF];
#pragma unroll
    for (int k = 0; k < PF; k++) {
        pidx[k] = (k * gridDim.x + blockIdx.x) * 16 + wave * 4 + slot;
        page[k] = pidx[k] < pv.maxgp ? pt[pidx[k]] : -1;
    }
    const int N = pv.global_len[um];
    const int n_pages = (N + pv.P - 1) >> pv.logP;
    for (int i = threadIdx.x; i < G * pv.d; i += 256)
        s_q[i] = q_ld<DT>(a.q, ((size_t)b * pv.Hq + (size_t)h * G) * pv.d + i);
    __syncthreads();
    const int n_iter = (n_pages + gridDim.x * 16 - 1) / (gridDim.x * 16);  // the same for every lane: no divergence
    for (int it0 = 0; it0 < n_iter; it0 += PF) {
        float acc[G][PF];
#pragma unroll
        for (int g = 0; g < G; g++)
#pragma unroll
            for (int k = 0; k < PF; k++) acc[g][k] = 0.f;
        int cur_idx[PF], cur_page[PF];
#pragma unroll
        for (int k = 0; k < PF; k++) { cur_idx[k] = pidx[k]; cur_page[k] = (pidx[k] < n_pages && page[k] >= 0) ? page[k] : 0; }
        if (it0 + PF < n_iter) {  // the ids of the next turn, on their way while this one is read and summed
#pragma unroll
            for (int k = 0; k < PF; k++) {
                pidx[k] = ((it0 + PF + k) * gridDim.x + blockIdx.x) * 16 + wave * 4 + slot;
                page[k] = pidx[k] < pv.maxgp ? pt[pidx[k]] : -1;
            }
        }
        for (int c = sub; c < cpr; c += 16) {  // one turn for 256-byte rows
            uint4 lo4[PF], hi4[PF];
#pragma unroll
            for (int k = 0; k < PF; k++) {
                const char *lo_row = a.lm + (size_t)cur_page[k] * 2 * pv.row_bytes;
                lo4[k] = *reinterpret_cast<const uint4 *>(lo_row + c * 16);
                hi4[k] = *reinterpret_cast<const uint4 *>(lo_row + pv.row_bytes + c * 16);
            }
#pragma unroll
            for (int g = 0; g < G; g++) {
                const float *qg = s_q + g * pv.d + c * EPC;
                float qv[EPC];
#pragma unroll
                for (int i = 0; i < EPC; i++) qv[i] = qg[i];
#pragma unroll
                for (int k = 0; k < PF; k++) {
                    const uint32_t lw[4] = {lo4[k].x, lo4[k].y, lo4[k].z, lo4[k].w};
                    const uint32_t hw[4] = {hi4[k].x, hi4[k].y, hi4[k].z, hi4[k].w};
#pragma unroll
                    for (int i = 0; i < 4; i++) {
                        if (DT == WGKV_F32) {
                            acc[g][k] += fmaxf(qv[i] * __uint_as_float(lw[i]), qv[i] * __uint_as_float(hw[i]));
                        } else {
                            acc[g][k] += fmaxf(qv[2 * i] * __uint_as_float(lw[i] << 16), qv[2 * i] * __uint_as_float(hw[i] << 16));
                            acc[g][k] += fmaxf(qv[2 * i + 1] * __uint_as_float(lw[i] & 0xffff0000u),
                                               qv[2 * i + 1] * __uint_as_float(hw[i] & 0xffff0000u));
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int k = 0; k < PF; k++) {
            float best = -INFINITY;
#pragma unroll
            for (int g = 0; g < G; g++) best = fmaxf(best, group_sum<16>(acc[g][k]));
            if (it0 + k < n_iter && cur_idx[k] < n_pages && sub == 0) a.scores[(size_t)u * a.score_stride + cur_idx[k]] = best;
        }
    }
}

__device__ __forceinline__ uint32_t quest_key(float x) {  // ascending in this key = descending score
    const uint32_t v = __float_as_uint(x);
    return ~((v & 0x80000000u) ? ~v : (v | 0x80000000u));
}

// The `want` smallest keys among n (ties: lower index first): returns the key of the last one taken
// and how many entries with exactly that key are taken.  One block of 1024 threads; s_hist: 256, s_sel: 4,
// s_tmp: 20 ints.
__device__ __forceinline__ void block_radix_cut(const float *vals, int n, int want, unsigned *s_hist,
                                                unsigned *s_sel, int *s_tmp, uint32_t &cut, int &ties) {
    if (threadIdx.x == 0) { s_sel[0] = 0u; s_sel[1] = 0u; s_sel[2] = (unsigned)want; }
    for (int pass = 3; pass >= 0; pass--) {
        if (threadIdx.x < 256) s_hist[threadIdx.x] = 0u;
        __syncthreads();
        const unsigned prefix = s_sel[0], mask = s_sel[1];
        for (int j = threadIdx.x; j < n; j += 1024) {
            const uint32_t key = quest_key(vals[j]);
            if ((key & mask) == prefix) atomicAdd(&s_hist[(key >> (8 * pass)) & 255u], 1u);
        }
        __syncthreads();
        // the bin in which the running count reaches the rank: a block-wide prefix over the 256 bins
        {
            const unsigned w = s_sel[2];
            const int cnt = threadIdx.x < 256 ? (int)s_hist[threadIdx.x] : 0;
            int total;
            const int ex = block_excl_scan(cnt, s_tmp, &total);
            __syncthreads();  // everybody has read s_sel
            if (threadIdx.x < 256 && (unsigned)ex < w && w <= (unsigned)(ex + cnt)) {
                s_sel[0] = prefix | ((unsigned)threadIdx.x << (8 * pass));
                s_sel[1] = mask | (255u << (8 * pass));
                s_sel[2] = w - (unsigned)ex;
            }
        }
        __syncthreads();
    }
    cut = s_sel[0];
    ties = (int)s_sel[2];
}

__global__ __launch_bounds__(1024) void quest_select_kernel(View pv, CallSeqs cs, QuestArgs a) {
    __shared__ unsigned s_hist[256];
    __shared__ unsigned s_sel[4];
    __shared__ int s_tmp[20];
    const int u = blockIdx.x, b = u / pv.Hkv, h = u % pv.Hkv;
    const int um = unit_meta(pv, cs.sid[b], a.layer, h);
    const int n_pages = (pv.global_len[um] + pv.P - 1) >> pv.logP;
    int32_t *sel = a.sel_pages + (size_t)u * a.budget_pages;
    if (n_pages <= a.budget_pages) {  // block-uniform: everything fits the budget
        for (int p = threadIdx.x; p < n_pages; p += 1024) sel[p] = p;
        if (threadIdx.x == 0) a.sel_count[u] = n_pages;
        return;
    }
    const float *sc = a.scores + (size_t)u * a.score_stride;
    uint32_t cut;
    int ties_to_take;
    block_radix_cut(sc, n_pages, a.budget_pages, s_hist, s_sel, s_tmp, cut, ties_to_take);
    int ties_seen = 0, taken = 0;
    for (int p0 = 0; p0 < n_pages; p0 += 1024) {
        const int p = p0 + threadIdx.x;
        uint32_t key = 0xffffffffu;
        if (p < n_pages) key = quest_key(sc[p]);
        const int is_tie = (p < n_pages && key == cut) ? 1 : 0;
        int n_ties;
        const int tie_rank = ties_seen + block_excl_scan(is_tie, s_tmp, &n_ties);
        const int take = (p < n_pages && (key < cut || (is_tie && tie_rank < ties_to_take))) ? 1 : 0;
        int n_take;
        const int idx = block_excl_scan(take, s_tmp, &n_take);
        if (take) sel[taken + idx] = p;
        ties_seen += n_ties;
        taken += n_take;
    }
    if (threadIdx.x == 0) a.sel_count[u] = taken;  // = budget_pages
}

size_t quest_landmark_bytes(const View &pv) {
    const size_t lm = (((size_t)pv.n_pages * 2 * pv.row_bytes) + 255) / 256 * 256;
    return lm + (((size_t)pv.S * pv.L * pv.Hkv * 4) + 255) / 256 * 256;
}

static void quest_split(const View &pv, void *landmarks, QuestArgs &a) {
    a.lm = (char *)landmarks;
    a.lm_len = (int32_t *)((char *)landmarks + (((size_t)pv.n_pages * 2 * pv.row_bytes) + 255) / 256 * 256);
}

hipError_t launch_quest_update(const View &pv, const CallSeqs &cs, int layer, void *landmarks, int reset,
                               hipStream_t st) {
    const int n_units = cs.n * pv.Hkv;
    QuestArgs a = {};
    a.layer = layer;
    a.reset = reset;
    quest_split(pv, landmarks, a);
    if (pv.row_bytes % 16 != 0) return hipErrorNotSupported;
    if (pv.dtype == WGKV_F32) hipLaunchKernelGGL(quest_update_kernel<WGKV_F32>, dim3(n_units), dim3(256), 0, st, pv, cs, a);
    else hipLaunchKernelGGL(quest_update_kernel<WGKV_BF16>, dim3(n_units), dim3(256), 0, st, pv, cs, a);
    return hipGetLastError();
}

hipError_t launch_quest_select(const View &pv, const CallSeqs &cs, int layer, const void *q, void *landmarks,
                               int budget_pages, float *scores, int64_t score_stride, int32_t *sel_pages,
                               int32_t *sel_count, int64_t max_pages, hipStream_t st) {
    const int n_units = cs.n * pv.Hkv;
    QuestArgs a = {};
    a.layer = layer;
    quest_split(pv, landmarks, a);
    a.q = (const char *)q;
    a.scores = scores;
    a.score_stride = score_stride;
    a.budget_pages = budget_pages;
    a.sel_pages = sel_pages;
    a.sel_count = sel_count;
    // 16 pages per block and turn, four turns in flight: enough blocks for one pass of four turns where the
    // launch stays within a few rounds of resident blocks, more turns per block beyond that
    int bx = (int)((max_pages + 63) / 64);
    const int cap = n_units > 0 ? (4096 / n_units > 1 ? 4096 / n_units : 1) : 1;
    bx = bx < 1 ? 1 : (bx > cap ? cap : bx);
    const dim3 grid(bx, n_units);
    const size_t smem = (size_t)pv.G * pv.d * sizeof(float);
#define WGKV_QS(DT_, G_) hipLaunchKernelGGL((quest_score_kernel<DT_, G_>), grid, dim3(256), smem, st, pv, cs, a)
    if (pv.dtype == WGKV_F32) {
        if (pv.G == 1) WGKV_QS(WGKV_F32, 1); else if (pv.G == 2) WGKV_QS(WGKV_F32, 2);
        else if (pv.G == 4) WGKV_QS(WGKV_F32, 4); else if (pv.G == 8) WGKV_QS(WGKV_F32, 8);
        else return hipErrorNotSupported;
    } else {
        if (pv.G == 1) WGKV_QS(WGKV_BF16, 1); else if (pv.G == 2) WGKV_QS(WGKV_BF16, 2);
        else if (pv.G == 4) WGKV_QS(WGKV_BF16, 4); else if (pv.G == 8) WGKV_QS(WGKV_BF16, 8);
        else return hipErrorNotSupported;
    }
#undef WGKV_QS
    hipLaunchKernelGGL(quest_select_kernel, dim3(n_units), dim3(1024), 0, st, pv, cs, a);
    return hipGetLastError();
}

}  // namespace wgkv
