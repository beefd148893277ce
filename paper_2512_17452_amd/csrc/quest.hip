// Read-time page selection over the admitted cache (appendix "Synergy with KV Selection":
// Quest-style selection with key landmarks, the per-page minimum and maximum key vectors).
//
//  quest_update_kernel   landmarks of the pages that changed since the last update
//  quest_score_kernel    criticality of every page for a decode query:
//                        U_p = max over the group of sum_e max(q[e] lo_p[e], q[e] hi_p[e])
//  quest_select_kernel   the budget's worth of pages with the largest U, as ascending indices
//
// Landmarks are stored per (sequence slot, layer, kv head) and page of its global cache in cache order, in the
// pool's dtype (a minimum or maximum of stored values is a stored value):
// [S * L * Hkv][max_global_pages_per_head][lo row, hi row][d], followed by one int32 per head: the number of
// entries its landmarks cover.  A head's landmarks are contiguous and found without its page table, so scoring
// has no dependent load in front of its stream (stored by physical page, as a first version had them, the
// scoring kernel waited for the page ids first and read 512-byte pieces scattered over the pool).
#include "wgkv_dev.h"

namespace wgkv {

struct QuestArgs {
    int layer;
    int reset;               // recompute every page of the given heads
    char *lm;                // landmarks [S * L * Hkv][maxgp][2][d] of the pool dtype
    int32_t *lm_len;         // [S * L * Hkv]
    const char *q;           // [n_seqs][Hq][d]
    float *scores;           // [n_units][score_stride]
    long long score_stride;
    int budget_pages;
    int32_t *sel_pages;      // [n_units][budget_pages]
    int32_t *sel_count;      // [n_units]
};

// How many blocks of quest_score_bf16_kernel work on each (sequence, kv head) unit of a call: from the host's
// bounds of the heads' lengths, so that a block knows its head and its pages without reading device memory.
struct QuestPlan {
    uint8_t nb[kMaxCallUnits];
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
        char *lo_row = a.lm + ((size_t)um * pv.maxgp + p) * 2 * pv.row_bytes, *hi_row = lo_row + pv.row_bytes;
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

// The general form, launched for fp32 pools (bf16 pools take quest_score_bf16_kernel below).
// Sixteen lanes per page, four pages per wave at a time and four such turns in flight; a lane reads 16 bytes
// of the minimum row and of the maximum row of a page, once for the whole group of query heads, whose queries sit
// in LDS as floats.  The launch is small (1/P of the keys), so its time is what stands in front of its stream:
// a head's landmarks are addressed by page index alone, so the loads of the first turn go out at once, together
// with the requests for the head's length and the queries (they stay inside the head's maxgp pages whatever the
// length is; what lies past the last page is read and dropped), and the loads of a turn are in flight while
// the turn before it is summed.  The grid is sized so that nearly every lane group has a single turn of four pages.
template <int DT, int G>
__global__ __launch_bounds__(256) void quest_score_kernel(View pv, CallSeqs cs, QuestArgs a) {
    extern __shared__ float s_q[];  // [G][d]
    constexpr int EPC = DT == WGKV_F32 ? 4 : 8;  // elements per 16-byte chunk
    constexpr int PF = 4;
    const int u = blockIdx.y, b = u / pv.Hkv, h = u % pv.Hkv;
    const int um = unit_meta(pv, cs.sid[b], a.layer, h);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane & 15, slot = lane >> 4, cpr = (int)(pv.row_bytes / 16);
    const int n_c = (cpr + 15) >> 4;  // turns over a row: one for rows of up to 256 bytes
    const char *lm = a.lm + (size_t)um * pv.maxgp * 2 * pv.row_bytes;
    const int first = blockIdx.x * 16 + wave * 4 + slot, stride = gridDim.x * 16;
    uint4 lo_n[PF], hi_n[PF];
    // the pages first + (it + k) * stride, chunk sub + 16 * ci of their two rows; indices are clamped into the
    // head's part of the buffer, the sums of clamped ones are not used
    auto request = [&](int it, int ci) {
        const int c = min(sub + 16 * ci, cpr - 1);
#pragma unroll
        for (int k = 0; k < PF; k++) {
            const int idx = min(first + (it + k) * stride, pv.maxgp - 1);
            const char *lo_row = lm + (size_t)idx * 2 * pv.row_bytes + c * 16;
            lo_n[k] = load_once16(lo_row);
            hi_n[k] = load_once16(lo_row + pv.row_bytes);
        }
    };
    const int N = pv.global_len[um];
    const size_t q0 = ((size_t)b * pv.Hq + (size_t)h * G) * pv.d;
    float qx[4];  // group size <= 8, head_dim <= 128: at most four elements per thread, requested together
#pragma unroll
    for (int j = 0; j < 4; j++)  // no branch around a load: they stay in flight together
        qx[j] = q_ld<DT>(a.q, q0 + min(j * 256 + (int)threadIdx.x, G * pv.d - 1));
    request(0, 0);
#pragma unroll
    for (int j = 0; j < 4; j++)
        if (j * 256 + (int)threadIdx.x < G * pv.d) s_q[j * 256 + threadIdx.x] = qx[j];
    __syncthreads();
    // never past the caller's score row, whatever the device's length is (the host sized the row from its own bound)
    const int n_pages = (int)min((long long)((N + pv.P - 1) >> pv.logP), a.score_stride);
    const int n_iter = (n_pages + stride - 1) / stride;  // the same for every lane: no divergence
    for (int it0 = 0; it0 < n_iter; it0 += PF) {
        float acc[G][PF];
#pragma unroll
        for (int g = 0; g < G; g++)
#pragma unroll
            for (int k = 0; k < PF; k++) acc[g][k] = 0.f;
        for (int ci = 0; ci < n_c; ci++) {
            uint4 lo4[PF], hi4[PF];
#pragma unroll
            for (int k = 0; k < PF; k++) { lo4[k] = lo_n[k]; hi4[k] = hi_n[k]; }
            const int ci_n = ci + 1 < n_c ? ci + 1 : 0, it_n = ci + 1 < n_c ? it0 : it0 + PF;
            if (it_n < n_iter) request(it_n, ci_n);
            const int c = sub + 16 * ci;
            if (c < cpr) {
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
        }
#pragma unroll
        for (int k = 0; k < PF; k++) {
            float best = -INFINITY;
#pragma unroll
            for (int g = 0; g < G; g++) best = fmaxf(best, group_sum<16>(acc[g][k]));
            const int idx = first + (it0 + k) * stride;
            if (it0 + k < n_iter && idx < n_pages && sub == 0) a.scores[(size_t)u * a.score_stride + idx] = best;
        }
    }
}

// The same for bf16 pools, whose rows are at most 256 bytes (one 16-byte chunk per lane).  max(q lo, q hi) equals
// q * (hi where q >= 0, else lo) exactly, because hi >= lo and a product of two bf16 values is exact in fp32: one
// bit-select per word, with a mask made once from the signs of the query, then the two-element dot product on the
// packed pairs.  The queries stay packed in the registers of the lanes that use them: no LDS and no barrier, so
// the landmarks, the queries and the head's length are one round trip.
// Work split: a head's pages in groups of 64 (four waves x four lane groups x four loads in flight); the head has
// plan.nb[u] blocks (launched: the largest of them for every head, the surplus returns at once), block j takes
// the groups j, j + nb, ...  The host sizes nb from its bounds of the lengths so that the launch is one round of
// resident blocks with equal turns; the loop itself runs to the length on the device, so a bound that is stale
// (a replayed graph) costs turns, not pages.
typedef __attribute__((ext_vector_type(2))) __bf16 quest_bf16x2_t;
template <int G>
__global__ __launch_bounds__(256) void quest_score_bf16_kernel(View pv, CallSeqs cs, QuestArgs a, QuestPlan plan) {
    constexpr int PF = 4;
    const int u = blockIdx.y, nb = plan.nb[u];
    if ((int)blockIdx.x >= nb) return;
    const int b = u / pv.Hkv, h = u % pv.Hkv;
    const int um = unit_meta(pv, cs.sid[b], a.layer, h);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane & 15, slot = lane >> 4, cpr = (int)(pv.row_bytes / 16);
    const int c = min(sub, cpr - 1);  // lanes past the end of a short row read its last chunk and add nothing
    const char *lm = a.lm + (size_t)um * pv.maxgp * 2 * pv.row_bytes;
    const int first = blockIdx.x * 64 + wave * 4 + slot, stride = nb * 64;
    uint4 lo_n[PF], hi_n[PF];
    auto request = [&](int it) {  // pages first + it * stride + 16 k, clamped into the head's part of the buffer
#pragma unroll
        for (int k = 0; k < PF; k++) {
            const int idx = min(first + it * stride + 16 * k, pv.maxgp - 1);
            const char *lo_row = lm + (size_t)idx * 2 * pv.row_bytes + c * 16;
            lo_n[k] = load_once16(lo_row);
            hi_n[k] = load_once16(lo_row + pv.row_bytes);
        }
    };
    const int N = pv.global_len[um];
    uint32_t qw[G][4], qm[G][4];
#pragma unroll
    for (int g = 0; g < G; g++) {
        const uint4 x = *reinterpret_cast<const uint4 *>(a.q + (((size_t)b * pv.Hq + (size_t)h * G + g) * pv.d) * 2 + c * 16);
        qw[g][0] = x.x; qw[g][1] = x.y; qw[g][2] = x.z; qw[g][3] = x.w;
    }
    request(0);
#pragma unroll
    for (int g = 0; g < G; g++)
#pragma unroll
        for (int i = 0; i < 4; i++) {
            const uint32_t w = sub < cpr ? qw[g][i] : 0u;
            qw[g][i] = w;
            qm[g][i] = ((w & 0x8000u) ? 0u : 0xffffu) | ((w & 0x80000000u) ? 0u : 0xffff0000u);  // all ones where q >= 0
        }
    // never past the caller's score row, whatever the device's length is (the host sized the row from its own bound)
    const int n_pages = (int)min((long long)((N + pv.P - 1) >> pv.logP), a.score_stride);
    for (int it = 0; (int)blockIdx.x * 64 + it * stride < n_pages; it++) {  // block-uniform
        uint32_t lw[PF][4], hw[PF][4];
#pragma unroll
        for (int k = 0; k < PF; k++) {
            lw[k][0] = lo_n[k].x; lw[k][1] = lo_n[k].y; lw[k][2] = lo_n[k].z; lw[k][3] = lo_n[k].w;
            hw[k][0] = hi_n[k].x; hw[k][1] = hi_n[k].y; hw[k][2] = hi_n[k].z; hw[k][3] = hi_n[k].w;
        }
        if ((int)blockIdx.x * 64 + (it + 1) * stride < n_pages) request(it + 1);
#pragma unroll
        for (int k = 0; k < PF; k++) {
            float best = -INFINITY;
#pragma unroll
            for (int g = 0; g < G; g++) {
                float d = 0.f;
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    const uint32_t pick = (hw[k][i] & qm[g][i]) | (lw[k][i] & ~qm[g][i]);
                    d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(quest_bf16x2_t, pick),
                                                        __builtin_bit_cast(quest_bf16x2_t, qw[g][i]), d, false);
                }
                best = fmaxf(best, group_sum<16>(d));
            }
            const int idx = first + it * stride + 16 * k;
            if (idx < n_pages && sub == 0) a.scores[(size_t)u * a.score_stride + idx] = best;
        }
    }
}

__device__ __forceinline__ uint32_t quest_key(float x) {  // ascending in this key = descending score
    const uint32_t v = __float_as_uint(x);
    return ~((v & 0x80000000u) ? ~v : (v | 0x80000000u));
}

// One block of 256 threads per head.  Thread t owns the scores [16 t, 16 t + 16) of every stretch of 4096, so the
// page order is the thread order and the picked indices come out ascending from two block-wide prefixes (ties
// before the thread's own, picks before the thread's own).  The first stretch is requested at once, together
// with the head's length (a score row is score_stride wide, so nothing outside it is read whatever the length),
// and kept as keys in registers for the four radix passes; longer heads read the rest from memory in every pass.
constexpr int kSelThreads = 256, kSelOwn = 16, kSelStretch = kSelThreads * kSelOwn;

// The `want` smallest keys among n (ties: lower index first): the key of the last one taken and how many entries
// with exactly that key are taken.  kreg: this thread's keys of the first stretch.  s_hist: 256, s_sel: 4, s_tmp: 20 ints.
__device__ __forceinline__ void block_radix_cut(const float *vals, const uint32_t (&kreg)[kSelOwn], int n, int want,
                                                unsigned *s_hist, unsigned *s_sel, int *s_tmp, uint32_t &cut, int &ties) {
    if (threadIdx.x == 0) { s_sel[0] = 0u; s_sel[1] = 0u; s_sel[2] = (unsigned)want; }
    const int own0 = threadIdx.x * kSelOwn;
    for (int pass = 3; pass >= 0; pass--) {
        s_hist[threadIdx.x] = 0u;
        __syncthreads();
        const unsigned prefix = s_sel[0], mask = s_sel[1];
#pragma unroll
        for (int i = 0; i < kSelOwn; i++)
            if (own0 + i < n && (kreg[i] & mask) == prefix) atomicAdd(&s_hist[(kreg[i] >> (8 * pass)) & 255u], 1u);
        for (int j = kSelStretch + threadIdx.x; j < n; j += kSelThreads) {
            const uint32_t key = quest_key(vals[j]);
            if ((key & mask) == prefix) atomicAdd(&s_hist[(key >> (8 * pass)) & 255u], 1u);
        }
        __syncthreads();
        // the bin in which the running count reaches the rank: a block-wide prefix over the 256 bins
        const unsigned w = s_sel[2];
        const int cnt = (int)s_hist[threadIdx.x];
        int total;
        const int ex = block_excl_scan(cnt, s_tmp, &total);
        __syncthreads();  // everybody has read s_sel
        if ((unsigned)ex < w && w <= (unsigned)(ex + cnt)) {
            s_sel[0] = prefix | ((unsigned)threadIdx.x << (8 * pass));
            s_sel[1] = mask | (255u << (8 * pass));
            s_sel[2] = w - (unsigned)ex;
        }
        __syncthreads();
    }
    cut = s_sel[0];
    ties = (int)s_sel[2];
}

__global__ __launch_bounds__(kSelThreads) void quest_select_kernel(View pv, CallSeqs cs, QuestArgs a) {
    __shared__ unsigned s_hist[256];
    __shared__ unsigned s_sel[4];
    __shared__ int s_tmp[20];
    const int u = blockIdx.x, b = u / pv.Hkv, h = u % pv.Hkv;
    const int um = unit_meta(pv, cs.sid[b], a.layer, h);
    const float *sc = a.scores + (size_t)u * a.score_stride;
    const int own0 = threadIdx.x * kSelOwn;
    const int N = pv.global_len[um];
    uint32_t kreg[kSelOwn];
#pragma unroll
    for (int i = 0; i < kSelOwn; i++)  // clamped, not skipped: no branch around a load, the sixteen are in flight together
        kreg[i] = quest_key(sc[min((long long)(own0 + i), a.score_stride - 1)]);
    const int n_pages = (int)min((long long)((N + pv.P - 1) >> pv.logP), a.score_stride);  // what was scored
    int32_t *sel = a.sel_pages + (size_t)u * a.budget_pages;
    if (n_pages <= a.budget_pages) {  // block-uniform: everything fits the budget
        for (int p = threadIdx.x; p < n_pages; p += kSelThreads) sel[p] = p;
        if (threadIdx.x == 0) a.sel_count[u] = n_pages;
        return;
    }
    uint32_t cut;
    int ties_to_take;
    block_radix_cut(sc, kreg, n_pages, a.budget_pages, s_hist, s_sel, s_tmp, cut, ties_to_take);
    int ties_seen = 0, taken = 0;
    for (int p0 = 0; p0 < n_pages; p0 += kSelStretch) {
        if (p0 > 0) {
#pragma unroll
            for (int i = 0; i < kSelOwn; i++) kreg[i] = quest_key(sc[min(p0 + own0 + i, n_pages - 1)]);
        }
        int my_ties = 0;
#pragma unroll
        for (int i = 0; i < kSelOwn; i++) my_ties += (p0 + own0 + i < n_pages && kreg[i] == cut) ? 1 : 0;
        int n_ties;
        int tie_rank = ties_seen + block_excl_scan(my_ties, s_tmp, &n_ties);
        unsigned take_bits = 0u;
        int my_take = 0;
#pragma unroll
        for (int i = 0; i < kSelOwn; i++) {
            const bool in = p0 + own0 + i < n_pages, is_tie = in && kreg[i] == cut;
            const bool take = in && (kreg[i] < cut || (is_tie && tie_rank < ties_to_take));
            tie_rank += is_tie ? 1 : 0;
            take_bits |= take ? (1u << i) : 0u;
            my_take += take ? 1 : 0;
        }
        int n_take;
        int at = taken + block_excl_scan(my_take, s_tmp, &n_take);
#pragma unroll
        for (int i = 0; i < kSelOwn; i++)
            if (take_bits & (1u << i)) sel[at++] = p0 + own0 + i;
        ties_seen += n_ties;
        taken += n_take;
    }
    if (threadIdx.x == 0) a.sel_count[u] = taken;  // = budget_pages
}

static size_t quest_rows_bytes(const View &pv) {
    return (((size_t)pv.S * pv.L * pv.Hkv * pv.maxgp * 2 * pv.row_bytes) + 255) / 256 * 256;
}

size_t quest_landmark_bytes(const View &pv) {
    return quest_rows_bytes(pv) + (((size_t)pv.S * pv.L * pv.Hkv * 4) + 255) / 256 * 256;
}

static void quest_split(const View &pv, void *landmarks, QuestArgs &a) {
    a.lm = (char *)landmarks;
    a.lm_len = (int32_t *)((char *)landmarks + quest_rows_bytes(pv));
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
                               int32_t *sel_count, const int32_t *len_ub, hipStream_t st) {
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
    int64_t max_pages = 0, total_groups = 0;  // from the host's bounds len_ub[n_units] of the heads' lengths
    for (int u = 0; u < n_units; u++) {
        const int64_t pages = ((int64_t)len_ub[u] + pv.P - 1) >> pv.logP;
        max_pages = max_pages > pages ? max_pages : pages;
        total_groups += (pages + 63) / 64;
    }
    if (pv.dtype == WGKV_BF16) {
        // at most about kQuestBlocks blocks in all, every block with the same number of turns: one turn each while
        // the call has no more than that many groups (measured on 60K pages in 64 heads: 320 / 640 / 960 / 1280
        // blocks allowed: 12.5 / 11.7 / 11.1 / 10.6 us)
        constexpr int64_t kQuestBlocks = 1280;
        const int64_t turns = total_groups > kQuestBlocks ? (total_groups + kQuestBlocks - 1) / kQuestBlocks : 1;
        QuestPlan plan;
        int bx = 1;
        for (int u = 0; u < n_units; u++) {
            const int64_t groups = ((((int64_t)len_ub[u] + pv.P - 1) >> pv.logP) + 63) / 64;
            int64_t nb = (groups + turns - 1) / turns;
            nb = nb < 1 ? 1 : (nb > 255 ? 255 : nb);
            plan.nb[u] = (uint8_t)nb;
            bx = bx > (int)nb ? bx : (int)nb;
        }
        const dim3 grid(bx, n_units);
#define WGKV_QB(G_) hipLaunchKernelGGL((quest_score_bf16_kernel<G_>), grid, dim3(256), 0, st, pv, cs, a, plan)
        if (pv.G == 1) WGKV_QB(1); else if (pv.G == 2) WGKV_QB(2);
        else if (pv.G == 4) WGKV_QB(4); else if (pv.G == 8) WGKV_QB(8);
        else return hipErrorNotSupported;
#undef WGKV_QB
    } else {
        // 16 pages per block and turn, four turns in flight: enough blocks for one pass of four turns where the
        // launch stays within a few rounds of resident blocks, more turns per block beyond that
        int bx = (int)((max_pages + 63) / 64);
        const int cap = n_units > 0 ? (512 / n_units > 1 ? 512 / n_units : 1) : 1;
        bx = bx < 1 ? 1 : (bx > cap ? cap : bx);
        const dim3 grid(bx, n_units);
        const size_t smem = (size_t)pv.G * pv.d * sizeof(float);
#define WGKV_QS(G_) hipLaunchKernelGGL((quest_score_kernel<WGKV_F32, G_>), grid, dim3(256), smem, st, pv, cs, a)
        if (pv.G == 1) WGKV_QS(1); else if (pv.G == 2) WGKV_QS(2);
        else if (pv.G == 4) WGKV_QS(4); else if (pv.G == 8) WGKV_QS(8);
        else return hipErrorNotSupported;
#undef WGKV_QS
    }
    hipLaunchKernelGGL(quest_select_kernel, dim3(n_units), dim3(kSelThreads), 0, st, pv, cs, a);
    return hipGetLastError();
}

}  // namespace wgkv
