// Admission, paging and promotion kernels for gfx950 (wave64).
//
//  init_kernel            free stack + cleared tables                       (Sec. 4.1)
//  prefill_count_kernel   gate score -> admit mask, per-block admitted counts (Sec. 3.3 last sentence)
//  prefill_plan_kernel    prefix sums over blocks and units, page hand-out    (Sec. 4.1, 4.2)
//  prefill_scatter_kernel stable compaction of admitted K/V rows into global pages, then the
//                         last min(W,T) tokens into the ring                  (Sec. 4.2)
//  decode_step_kernel     lazy promotion of the victim, then overwrite        (Sec. 4.3 (1)-(3))
//  decode_promote_kernel, decode_promote_move_kernel
//                         steps (1)-(2) of every layer ahead of the layers' ring writes
//  decode_ring_kernel     step (3) alone, for units promoted ahead
//  free_seq_kernel        pages of a sequence slot back to the free stack
//
// Page hand-out never races: demands are prefix-summed in (sequence position in
// the call, kv head) order and unit u takes free_stack[top-1-base_u-i].
#include "wgkv_dev.h"

namespace wgkv {

constexpr int kPrefillBlk = 512;   // leaving tokens per block of 256 threads
constexpr int kTok = kPrefillBlk / 256;  // tokens per thread
constexpr int kPlanThreads = 1024; // the one block of prefill_plan_kernel

struct PrefillArgs {
    int layer;
    int nblk_max;         // blocks of leaving tokens per unit (the row stride of cnt)
    int max_adm;          // the caller's bound on tokens admitted per unit in this call, < 0: none
    float tau;
    const char *k, *v;    // [sumT][Hkv][d]
    const float *g;       // [sumT][Hkv]
    uint8_t *admit_out;   // optional
    int32_t *cnt;         // [n_units][nblk_max] admitted per block -> exclusive offsets
    int32_t *plan;        // [0]=abort flag, [1+u]=G_old of unit u
};

struct DecodeArgs {
    int layer;
    float tau;
    const char *k, *v;    // [n_seqs][Hkv][d]
    const float *g;       // [n_seqs][Hkv]
    uint8_t *promoted_out;
};

__global__ void init_kernel(View pv) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    const size_t i0 = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t n_sl = (size_t)pv.S * pv.L, n_u = n_sl * pv.Hkv;
    for (size_t i = i0; i < (size_t)pv.n_pages; i += stride) pv.free_stack[i] = pv.n_pages - 1 - (int32_t)i;
    for (size_t i = i0; i < n_sl; i += stride) pv.seq_len[i] = 0;
    for (size_t i = i0; i < n_u; i += stride) pv.global_len[i] = 0;
    for (size_t i = i0; i < n_u * pv.nlp; i += stride) pv.local_pt[i] = -1;
    for (size_t i = i0; i < n_u * pv.maxgp; i += stride) pv.global_pt[i] = -1;
    for (size_t i = i0; i < n_u * pv.W; i += stride) pv.ring_g[i] = 0.0f;
    for (size_t i = i0; i < (size_t)kMaxCallUnits; i += stride) pv.unit_counters[i] = 0;
    for (size_t i = i0; i < n_u; i += stride) pv.ahead[i] = -1;
    // the pool starts as zeros (no kernel relies on it: rows past a head's last token are never read)
    uint4 *pool16 = reinterpret_cast<uint4 *>(pv.pool);
    const size_t n16 = (size_t)pv.n_pages * pv.page_bytes / 16;
    for (size_t i = i0; i < n16; i += stride) pool16[i] = make_uint4(0u, 0u, 0u, 0u);
    if (i0 == 0) { *pv.free_top = pv.n_pages; *pv.err_flag = 0; }
}

// Score of leaving position p of a unit: from the ring if the token was fed by
// an earlier call, else from this call's scores.
__device__ __forceinline__ float leaving_score(const View &pv, const PrefillArgs &a, int um, int h,
                                               int p, int t0, int base) {
    if (p < t0) return pv.ring_g[(size_t)um * pv.W + (p % pv.W)];
    return a.g[(size_t)(base + p - t0) * pv.Hkv + h];
}

__global__ __launch_bounds__(256) void prefill_count_kernel(View pv, CallSeqs cs, PrefillArgs a) {
    __shared__ int s_w[4];
    const int u = blockIdx.y, b = u / pv.Hkv, h = u % pv.Hkv;
    const int t0 = cs.t0[b], T = cs.ntok[b], base = cs.base[b];
    const int um = unit_meta(pv, cs.sid[b], a.layer, h);
    const int lo = max(0, t0 - pv.W), hi = max(0, t0 + T - pv.W), n_leave = hi - lo;
    const int i0 = blockIdx.x * kPrefillBlk + threadIdx.x * kTok;
    if (a.admit_out) {
#pragma unroll
        for (int j = 0; j < kTok; j++) {
            int i = i0 + j;
            if (i < T) {
                size_t row = (size_t)(base + i) * pv.Hkv + h;
                a.admit_out[row] = (uint8_t)(a.g[row] >= a.tau);
            }
        }
    }
    if (blockIdx.x * kPrefillBlk >= n_leave) return;  // block-uniform
    int c = 0;
#pragma unroll
    for (int j = 0; j < kTok; j++) {
        int i = i0 + j;
        if (i < n_leave) c += (int)(leaving_score(pv, a, um, h, lo + i, t0, base) >= a.tau);
    }
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    c = wave_incl_scan(c, lane);
    if (lane == 63) s_w[w] = c;
    __syncthreads();
    if (threadIdx.x == 0) a.cnt[(size_t)u * a.nblk_max + blockIdx.x] = s_w[0] + s_w[1] + s_w[2] + s_w[3];
}

__global__ __launch_bounds__(kPlanThreads) void prefill_plan_kernel(View pv, CallSeqs cs, PrefillArgs a) {
    __shared__ int s_adm[kMaxCallUnits];
    __shared__ int s_gold[kMaxCallUnits];
    __shared__ int s_base[kMaxCallUnits];
    __shared__ int s_dl[kMaxCallUnits];
    __shared__ int s_um[kMaxCallUnits];
    __shared__ int s_tmp[20];
    __shared__ int s_err, s_over;
    const int n_units = cs.n * pv.Hkv;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    constexpr int NW = kPlanThreads / 64;
    if (threadIdx.x == 0) { s_err = 0; s_over = 0; }
    // what phase B needs of the first kPlanThreads units is asked for now: the kernel is a
    // chain of round trips on cold metadata, and these do not depend on phase A
    int um0 = 0, gold0 = 0, lp00 = 0;
    if ((int)threadIdx.x < n_units) {
        um0 = unit_meta(pv, cs.sid[threadIdx.x / pv.Hkv], a.layer, threadIdx.x % pv.Hkv);
        gold0 = pv.global_len[um0];
        lp00 = pv.local_pt[(size_t)um0 * pv.nlp];
    }
    const int top = *pv.free_top;
    __syncthreads();
    // A: one wave per unit turns block counts into exclusive offsets
    for (int u = w; u < n_units; u += NW) {
        const int b = u / pv.Hkv;
        const int t0 = cs.t0[b], T = cs.ntok[b];
        const int n_leave = max(0, t0 + T - pv.W) - max(0, t0 - pv.W);
        const int nblk = (n_leave + kPrefillBlk - 1) / kPrefillBlk;
        int32_t *c = a.cnt + (size_t)u * a.nblk_max;
        int run = 0;
        for (int i0 = 0; i0 < nblk; i0 += 64) {
            int i = i0 + lane;
            int v = i < nblk ? c[i] : 0;
            int inc = wave_incl_scan(v, lane);
            if (i < nblk) c[i] = run + inc - v;
            run += __shfl(inc, 63);
        }
        if (lane == 0) {
            s_adm[u] = run;
            if (a.max_adm >= 0 && run > a.max_adm) s_over = 1;  // more admitted than the caller sized its pool for
        }
    }
    __syncthreads();
    // B: page demand of every unit, prefix over units in call order
    int carry = 0;
    for (int u0 = 0; u0 < n_units; u0 += kPlanThreads) {
        const int u = u0 + threadIdx.x;
        int demand = 0;
        if (u < n_units) {
            const int b = u / pv.Hkv, h = u % pv.Hkv;
            const int um = u0 == 0 ? um0 : unit_meta(pv, cs.sid[b], a.layer, h);
            const int gold = u0 == 0 ? gold0 : pv.global_len[um];
            const int lp0 = u0 == 0 ? lp00 : pv.local_pt[(size_t)um * pv.nlp];
            const int gnew = gold + s_adm[u];
            const int dl = (cs.ntok[b] > 0 && lp0 < 0) ? pv.nlp : 0;
            const int pages_new = (gnew + pv.P - 1) >> pv.logP;
            if (pages_new > pv.maxgp) s_err = WGKV_ERR_PT_OVERFLOW;
            demand = dl + pages_new - ((gold + pv.P - 1) >> pv.logP);
            s_gold[u] = gold;
            s_dl[u] = dl;
            s_um[u] = um;
        }
        int total;
        int ex = block_excl_scan(demand, s_tmp, &total);
        if (u < n_units) s_base[u] = carry + ex;
        carry += total;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        if (s_over) s_err = WGKV_ERR_ADMIT_BOUND;  // reported first: the host's page accounting relied on the bound
        else if (s_err == 0 && carry > top) s_err = WGKV_ERR_OUT_OF_PAGES;
    }
    __syncthreads();
    if (s_err != 0) {  // block-uniform: leave all state as it was
        if (threadIdx.x == 0) {
            a.plan[0] = 1;
            atomicCAS(pv.err_flag, 0, s_err);
        }
        return;
    }
    // C: page-table entries.  Page f of the call (in unit order) is free_stack[top-1-f] whatever
    // unit it goes to, so the hand-out is one flat loop over all threads, four loads in flight per
    // thread; the owner of f is the last unit whose base is <= f (units without demand share
    // their base with the next one and are never picked).
    for (int f0 = 0; f0 < carry; f0 += kPlanThreads * 4) {
        int pg[4];
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const int f = f0 + k * kPlanThreads + (int)threadIdx.x;
            pg[k] = pv.free_stack[top - 1 - min(f, carry - 1)];
        }
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const int f = f0 + k * kPlanThreads + (int)threadIdx.x;
            if (f < carry) {
                int lo_u = 0, hi_u = n_units - 1;  // invariant: s_base[lo_u] <= f
                while (lo_u < hi_u) {
                    const int mid = (lo_u + hi_u + 1) >> 1;
                    if (s_base[mid] <= f) lo_u = mid; else hi_u = mid - 1;
                }
                const int u = lo_u, i = f - s_base[u], dl = s_dl[u], um = s_um[u];
                if (i < dl) pv.local_pt[(size_t)um * pv.nlp + i] = pg[k];
                else pv.global_pt[(size_t)um * pv.maxgp + ((s_gold[u] + pv.P - 1) >> pv.logP) + (i - dl)] = pg[k];
            }
        }
    }
    // D: lengths
    for (int u = threadIdx.x; u < n_units; u += kPlanThreads) {
        const int b = u / pv.Hkv, h = u % pv.Hkv;
        const int um = unit_meta(pv, cs.sid[b], a.layer, h);
        pv.global_len[um] = s_gold[u] + s_adm[u];
        a.plan[1 + u] = s_gold[u];
    }
    for (int b = threadIdx.x; b < cs.n; b += kPlanThreads) pv.seq_len[cs.sid[b] * pv.L + a.layer] = cs.t0[b] + cs.ntok[b];
    if (threadIdx.x == 0) {
        *pv.free_top = top - carry;
        a.plan[0] = 0;
    }
}

constexpr int kScatterBatch = 8;  // rows a thread has in flight in the copy loop

// Row r of the new ring contents of a unit: token T - nr + r of the sequence's part of the call
// goes to slot (t0 + T - nr + r) mod W, its score with it.  lpr lanes of 16 bytes per row.
__device__ __forceinline__ void ring_put(const View &pv, const PrefillArgs &a, int um, int h, int base, int t0,
                                         int i, int sub) {
    const int slot = (t0 + i) % pv.W;
    const size_t row = (size_t)(base + i) * pv.Hkv + h;
    char *dp = page_ptr(pv, pv.local_pt[(size_t)um * pv.nlp + (slot >> pv.logP)]) +
               (size_t)(slot & (pv.P - 1)) * pv.row_bytes;
    *reinterpret_cast<uint4 *>(dp + sub * 16) = *reinterpret_cast<const uint4 *>(a.k + row * pv.row_bytes + sub * 16);
    *reinterpret_cast<uint4 *>(dp + pv.v_off + sub * 16) =
        *reinterpret_cast<const uint4 *>(a.v + row * pv.row_bytes + sub * 16);
    if (sub == 0) pv.ring_g[(size_t)um * pv.W + slot] = a.g[row];
}

// The copy is a chain of round trips if done row by row (page id, then the row, then the
// store), so the destination page ids of the block go to LDS once (its rows land in one
// contiguous range of the global cache) and a thread requests 8 rows before it stores any.
//
// The ring is rewritten in the same launch.  A ring slot whose old token leaves the window is read
// by exactly one block here (the one that owns the leaving token), so that block also writes the
// slot's new token, after a barrier behind its copy loop: every new ring token whose slot was
// occupied has such an owner (the occupant of a slot always leaves when a token of the call takes
// the slot).  Slots that were still empty (sequences shorter than the window) are written by the
// blocks past the first nblk_max of the grid, which read nothing from the ring.
__global__ __launch_bounds__(256) void prefill_scatter_kernel(View pv, CallSeqs cs, PrefillArgs a) {
    __shared__ int s_src[kPrefillBlk];  // admitted leaving tokens of the block, in order
    __shared__ int s_rpg[kPrefillBlk];  // ring page of the token if its row sits in the ring, else -1
    __shared__ int s_gp[kPrefillBlk];   // pages of the destination range
    __shared__ int s_tmp[20];
    if (a.plan[0] != 0) return;
    const int u = blockIdx.y, b = u / pv.Hkv, h = u % pv.Hkv;
    const int t0 = cs.t0[b], T = cs.ntok[b], base = cs.base[b];
    const int um = unit_meta(pv, cs.sid[b], a.layer, h);
    const int lo = max(0, t0 - pv.W), hi = max(0, t0 + T - pv.W), n_leave = hi - lo;
    if ((int)blockIdx.x >= a.nblk_max) {
        // new ring tokens whose slot held nothing: slot >= t0 while the ring is not full yet
        if (t0 >= pv.W) return;
        const int nr = min(T, pv.W), lpr = pv.row_bytes >> 4;
        const int r = (((int)blockIdx.x - a.nblk_max) * 256 + (int)threadIdx.x) / lpr;
        if (r >= nr) return;
        const int i = T - nr + r;
        if ((t0 + i) % pv.W >= t0) ring_put(pv, a, um, h, base, t0, i, threadIdx.x % lpr);
        return;
    }
    if (blockIdx.x * kPrefillBlk >= n_leave) return;
    const int dst0 = a.plan[1 + u] + a.cnt[(size_t)u * a.nblk_max + blockIdx.x];
    const int i0 = blockIdx.x * kPrefillBlk + threadIdx.x * kTok;
    int f[kTok], rpg[kTok], c = 0;
#pragma unroll
    for (int j = 0; j < kTok; j++) {
        int i = i0 + j;
        f[j] = (i < n_leave) ? (int)(leaving_score(pv, a, um, h, lo + i, t0, base) >= a.tau) : 0;
        rpg[j] = -1;
        if (f[j] && lo + i < t0)  // fed by an earlier call: the row sits in the ring
            rpg[j] = pv.local_pt[(size_t)um * pv.nlp + (((lo + i) % pv.W) >> pv.logP)];
        c += f[j];
    }
    int n_adm;
    int rank = block_excl_scan(c, s_tmp, &n_adm);
#pragma unroll
    for (int j = 0; j < kTok; j++)
        if (f[j]) {
            s_src[rank] = i0 + j;
            s_rpg[rank++] = rpg[j];
        }
    const int pg_first = dst0 >> pv.logP;
    const int n_pg = n_adm > 0 ? ((dst0 + n_adm - 1) >> pv.logP) - pg_first + 1 : 0;  // <= kPrefillBlk
    for (int i = threadIdx.x; i < n_pg; i += 256) s_gp[i] = pv.global_pt[(size_t)um * pv.maxgp + pg_first + i];
    __syncthreads();
    // copy the admitted rows: lpr lanes of 16 bytes per row, K and V
    const int lpr = pv.row_bytes >> 4;
    const int rows_per_pass = 256 / lpr;
    const int sub = threadIdx.x % lpr;
    const size_t sub16 = (size_t)sub * 16;
    auto src_of = [&](int r, const char *&ks, const char *&vs) __attribute__((always_inline)) {
        ks = a.k;  // a row past the end reads the first row of the call and drops it
        vs = a.v;
        if (r < n_adm) {
            const int p = lo + s_src[r], pgid = s_rpg[r];
            if (pgid >= 0) {
                const int slot = p % pv.W;
                ks = page_ptr(pv, pgid) + (size_t)(slot & (pv.P - 1)) * pv.row_bytes;
                vs = ks + pv.v_off;
            } else {
                const size_t row = ((size_t)(base + p - t0) * pv.Hkv + h) * pv.row_bytes;
                ks = a.k + row;
                vs = a.v + row;
            }
        }
    };
    auto put = [&](int r, const uint4 &kk, const uint4 &vv) __attribute__((always_inline)) {
        if (r < n_adm) {
            const int dst = dst0 + r;
            char *dp = page_ptr(pv, s_gp[(dst >> pv.logP) - pg_first]) + (size_t)(dst & (pv.P - 1)) * pv.row_bytes;
            *reinterpret_cast<uint4 *>(dp + sub16) = kk;
            *reinterpret_cast<uint4 *>(dp + pv.v_off + sub16) = vv;
        }
    };
    static_assert(kScatterBatch == 8, "the copy loop is written out for 8 rows");
    const int rp = rows_per_pass;
    for (int r0 = threadIdx.x / lpr; r0 < n_adm; r0 += rp * kScatterBatch) {
        const char *k0, *k1, *k2, *k3, *k4, *k5, *k6, *k7, *v0, *v1, *v2, *v3, *v4, *v5, *v6, *v7;
        src_of(r0, k0, v0); src_of(r0 + rp, k1, v1); src_of(r0 + 2 * rp, k2, v2); src_of(r0 + 3 * rp, k3, v3);
        src_of(r0 + 4 * rp, k4, v4); src_of(r0 + 5 * rp, k5, v5); src_of(r0 + 6 * rp, k6, v6); src_of(r0 + 7 * rp, k7, v7);
#define WGKV_LD(p) load_once16((p) + sub16)
        const uint4 a0 = WGKV_LD(k0), b0 = WGKV_LD(v0), a1 = WGKV_LD(k1), b1 = WGKV_LD(v1), a2 = WGKV_LD(k2),
                    b2 = WGKV_LD(v2), a3 = WGKV_LD(k3), b3 = WGKV_LD(v3), a4 = WGKV_LD(k4), b4 = WGKV_LD(v4),
                    a5 = WGKV_LD(k5), b5 = WGKV_LD(v5), a6 = WGKV_LD(k6), b6 = WGKV_LD(v6), a7 = WGKV_LD(k7),
                    b7 = WGKV_LD(v7);
#undef WGKV_LD
        put(r0, a0, b0); put(r0 + rp, a1, b1); put(r0 + 2 * rp, a2, b2); put(r0 + 3 * rp, a3, b3);
        put(r0 + 4 * rp, a4, b4); put(r0 + 5 * rp, a5, b5); put(r0 + 6 * rp, a6, b6); put(r0 + 7 * rp, a7, b7);
    }
    // The ring slots of this block's leaving tokens that sat in the ring (leaving index < t0 - lo): every row and
    // score the block takes from them has arrived (the stores above used them), for all its threads behind the
    // barrier.  The slot of position p gets the last position of the call that is congruent to p modulo W.
    // Like the copy above, not a chain of round trips per row: the page ids of the ring go to LDS once (s_gp is free
    // behind the barrier) and a thread requests four pieces of 16 bytes of K and of V before it stores any.
    const int i_lo = (int)blockIdx.x * kPrefillBlk;
    const int i_hi = min(i_lo + kPrefillBlk, min(n_leave, t0 - lo));
    if (i_lo >= i_hi) return;  // block-uniform
    __syncthreads();
    const bool pt_in_lds = pv.nlp <= kPrefillBlk;  // block-uniform
    if (pt_in_lds) {
        for (int i = threadIdx.x; i < pv.nlp; i += 256) s_gp[i] = pv.local_pt[(size_t)um * pv.nlp + i];
        __syncthreads();
    }
    const int n_items = (i_hi - i_lo) * lpr;
    // one piece: 16 bytes of K and of V of the token that takes the slot of leaving position lo + i_lo + c / lpr
    // (the last position of the call congruent to it modulo W), its score, the slot and the slot's page; a piece
    // past the end asks for the last one again and is not stored.  Plain variables, written out: an array of
    // them ends up in scratch memory.
    auto ask = [&](int c, uint4 &kk, uint4 &vv, float &gg, int &slot, int &pg) __attribute__((always_inline)) {
        c = min(c, n_items - 1);
        const int pos = lo + i_lo + c / lpr, sb = c % lpr;
        const int q = pos + pv.W * ((t0 + T - 1 - pos) / pv.W);
        const size_t row = (size_t)(base + q - t0) * pv.Hkv + h;
        kk = *reinterpret_cast<const uint4 *>(a.k + row * pv.row_bytes + sb * 16);
        vv = *reinterpret_cast<const uint4 *>(a.v + row * pv.row_bytes + sb * 16);
        gg = a.g[row];
        slot = pos % pv.W;
        pg = pt_in_lds ? s_gp[slot >> pv.logP] : pv.local_pt[(size_t)um * pv.nlp + (slot >> pv.logP)];
    };
    auto place = [&](int c, const uint4 &kk, const uint4 &vv, float gg, int slot, int pg) __attribute__((always_inline)) {
        if (c < n_items) {
            char *dst = page_ptr(pv, pg) + (size_t)(slot & (pv.P - 1)) * pv.row_bytes + (c % lpr) * 16;
            *reinterpret_cast<uint4 *>(dst) = kk;
            *reinterpret_cast<uint4 *>(dst + pv.v_off) = vv;
            if (c % lpr == 0) pv.ring_g[(size_t)um * pv.W + slot] = gg;
        }
    };
    for (int c0 = threadIdx.x; c0 < n_items; c0 += 256 * 4) {
        uint4 ka, kb, kc, kd, va, vb, vc, vd;
        float ga, gb, gc, gd;
        int sa, sb_, sc, sd, pa, pb, pc, pd;
        ask(c0, ka, va, ga, sa, pa); ask(c0 + 256, kb, vb, gb, sb_, pb);
        ask(c0 + 512, kc, vc, gc, sc, pc); ask(c0 + 768, kd, vd, gd, sd, pd);
        place(c0, ka, va, ga, sa, pa); place(c0 + 256, kb, vb, gb, sb_, pb);
        place(c0 + 512, kc, vc, gc, sc, pc); place(c0 + 768, kd, vd, gd, sd, pd);
    }
}

// One block does the whole step: decisions and page hand-out first (they need a
// prefix over units), then the row moves.  The kernel is a chain of memory round trips, so
// everything whose address is known early is asked for early: the new rows at once, the
// victim's score and the page of its ring slot at the slot the host expects (checked against
// the device's own token count, which decides), the page of the promotion target as soon as
// the global length is there.  The row moves then only wait for the victim's row.
__global__ __launch_bounds__(1024) void decode_step_kernel(View pv, CallSeqs cs, DecodeArgs a) {
    __shared__ int s_gold[kMaxCallUnits];   // G before the step, bit 31 = promote
    __shared__ int s_lpage[kMaxCallUnits];  // page of the ring slot that is overwritten
    __shared__ int s_gpage[kMaxCallUnits];  // page of global slot G (promoting units)
    __shared__ int s_t[kMaxCallSeqs];       // token counts before the step
    __shared__ int s_tmp[20];
    __shared__ int s_err;
    const int n_units = cs.n * pv.Hkv;
    const int lpr = pv.row_bytes >> 4, n_items = n_units * lpr;
    uint4 kn = make_uint4(0, 0, 0, 0), vn = kn;  // this thread's first chunk of the new rows
    if ((int)threadIdx.x < n_items) {
        const size_t row = (size_t)(threadIdx.x / lpr) * pv.row_bytes + (threadIdx.x % lpr) * 16;
        kn = *reinterpret_cast<const uint4 *>(a.k + row);
        vn = *reinterpret_cast<const uint4 *>(a.v + row);
    }
    const int t_seq = ((int)threadIdx.x < cs.n) ? pv.seq_len[cs.sid[threadIdx.x] * pv.L + a.layer] : 0;
    if (threadIdx.x == 0) s_err = 0;
    __syncthreads();
    const int top = *pv.free_top;
    const int u = threadIdx.x;  // n_units <= 1024 = blockDim.x
    int demand = 0, dl = 0, promote = 0, gold = 0, um = 0, slot = 0, lpage = -1, gpage = -1, ahead_mask = -1;
    if (u < n_units) {
        // the token count comes from device memory, not from the launch arguments, so that a
        // captured launch can be replayed: every replay is one more token
        const int b = u / pv.Hkv, h = u % pv.Hkv;
        um = unit_meta(pv, cs.sid[b], a.layer, h);
        const int slot_h = cs.t0[b] % pv.W;  // where the host's count puts the victim
        const int t = pv.seq_len[cs.sid[b] * pv.L + a.layer];
        gold = pv.global_len[um];
        const int lp0 = pv.local_pt[(size_t)um * pv.nlp];
        float rg = pv.ring_g[(size_t)um * pv.W + slot_h];
        lpage = pv.local_pt[(size_t)um * pv.nlp + (slot_h >> pv.logP)];
        slot = t % pv.W;
        if (slot != slot_h) {  // a replayed launch: the host's count is the one of the capture
            rg = pv.ring_g[(size_t)um * pv.W + slot];
            lpage = pv.local_pt[(size_t)um * pv.nlp + (slot >> pv.logP)];
        }
        // promoted ahead for this very token (wgkv_decode_promote): steps (1)-(2) are done, only the mask is left
        const int ah = pv.ahead[um];
        const bool done = ah >= 0 && (ah >> 1) == t;
        ahead_mask = done ? (ah & 1) : -1;
        promote = !done && (t >= pv.W) && (rg >= a.tau);
        dl = (lp0 < 0) ? pv.nlp : 0;
        const int need = promote && ((gold & (pv.P - 1)) == 0);
        if (need && (gold >> pv.logP) >= pv.maxgp) s_err = WGKV_ERR_PT_OVERFLOW;
        else if (promote && !need) gpage = pv.global_pt[(size_t)um * pv.maxgp + (gold >> pv.logP)];
        demand = dl + need;
    }
    int total;
    const int ubase = block_excl_scan(demand, s_tmp, &total);
    if (total > top && threadIdx.x == 0 && s_err == 0) s_err = WGKV_ERR_OUT_OF_PAGES;
    __syncthreads();
    if (s_err != 0) {
        if (threadIdx.x == 0) atomicCAS(pv.err_flag, 0, s_err);
        return;
    }
    if (u < n_units) {
        for (int i = 0; i < dl; i++) {
            const int pg = pv.free_stack[top - 1 - (ubase + i)];
            pv.local_pt[(size_t)um * pv.nlp + i] = pg;
            if (i == (slot >> pv.logP)) lpage = pg;
        }
        if (demand > dl) {
            gpage = pv.free_stack[top - 1 - (ubase + dl)];
            pv.global_pt[(size_t)um * pv.maxgp + (gold >> pv.logP)] = gpage;
        }
        if (promote) pv.global_len[um] = gold + 1;
        if (a.promoted_out) a.promoted_out[u] = (uint8_t)(ahead_mask >= 0 ? ahead_mask : promote);
        s_gold[u] = (int)((unsigned)gold | ((unsigned)promote << 31));
        s_lpage[u] = lpage;
        s_gpage[u] = gpage;
    }
    if ((int)threadIdx.x < cs.n) {
        s_t[threadIdx.x] = t_seq;
        pv.seq_len[cs.sid[threadIdx.x] * pv.L + a.layer] = t_seq + 1;  // every unit thread has its copy already
    }
    if (threadIdx.x == 0) *pv.free_top = top - total;
    __syncthreads();  // the pages and counts of all units are in shared memory
    for (int c = threadIdx.x; c < n_items; c += blockDim.x) {
        const int uu = c / lpr, sub = c % lpr;
        const int b = uu / pv.Hkv, h = uu % pv.Hkv;
        const int m = unit_meta(pv, cs.sid[b], a.layer, h);
        const int sl = s_t[b] % pv.W;
        char *rp = page_ptr(pv, s_lpage[uu]) + (size_t)(sl & (pv.P - 1)) * pv.row_bytes + sub * 16;
        const int gi = s_gold[uu];
        if (gi < 0) {  // promote: ring row -> global slot G_old
            const int g0 = gi & 0x7fffffff;
            char *dp = page_ptr(pv, s_gpage[uu]) + (size_t)(g0 & (pv.P - 1)) * pv.row_bytes + sub * 16;
            const uint4 kk = *reinterpret_cast<const uint4 *>(rp);
            const uint4 vv = *reinterpret_cast<const uint4 *>(rp + pv.v_off);
            *reinterpret_cast<uint4 *>(dp) = kk;
            *reinterpret_cast<uint4 *>(dp + pv.v_off) = vv;
        }
        if (c != (int)threadIdx.x) {  // beyond the first 1024 chunks: not in registers yet
            const size_t row = (size_t)uu * pv.row_bytes + sub * 16;
            kn = *reinterpret_cast<const uint4 *>(a.k + row);
            vn = *reinterpret_cast<const uint4 *>(a.v + row);
        }
        *reinterpret_cast<uint4 *>(rp) = kn;
        *reinterpret_cast<uint4 *>(rp + pv.v_off) = vn;
        if (sub == 0) pv.ring_g[(size_t)m * pv.W + sl] = a.g[uu];
    }
}

// Steps (1)-(2) of Sec. 4.3 for every layer of the call's sequences at once, ahead of the layers' own
// decode steps: whether the victim of the coming token is promoted depends only on the score stored
// with it and on the token count, not on the layer's new K/V.  One block: the page hand-out needs a
// prefix over all units.  All-or-nothing like the step itself: a first sweep over the units only adds up
// the demand; the second takes the same decisions again (nothing they read has changed) and writes.
// A unit that was handled gets ahead[um] = (t << 1) | promoted; the rows are moved by
// decode_promote_move_kernel, and the layer's decode step then only writes the ring.
__device__ __forceinline__ void promote_decide(const View &pv, const CallSeqs &cs, float tau, int u, int &um, int &t,
                                               int &gold, int &promote, int &need) {
    // units in the order in which the layers' own steps would take their pages: layer, sequence of the call, head
    const int per_layer = cs.n * pv.Hkv;
    const int l = u / per_layer, r = u - l * per_layer;
    const int b = r / pv.Hkv;
    const int sl = cs.sid[b] * pv.L + l;
    um = sl * pv.Hkv + r % pv.Hkv;
    const int slot_h = cs.t0[b] % pv.W;  // where the host's count of the first layer puts the victim
    t = pv.seq_len[sl];
    const int ah = pv.ahead[um];
    gold = pv.global_len[um];
    float rg = pv.ring_g[(size_t)um * pv.W + slot_h];
    const int slot = t % pv.W;
    if (slot != slot_h) rg = pv.ring_g[(size_t)um * pv.W + slot];
    const bool done = ah >= 0 && (ah >> 1) == t;
    promote = done ? -1 : (int)((t >= pv.W) && (rg >= tau));
    need = promote > 0 && ((gold & (pv.P - 1)) == 0);
}

__global__ __launch_bounds__(1024) void decode_promote_kernel(View pv, CallSeqs cs, float tau) {
    __shared__ int s_tmp[20];
    __shared__ int s_err;
    const int n_all = cs.n * pv.L * pv.Hkv;
    const int top = *pv.free_top;
    if (threadIdx.x == 0) s_err = 0;
    __syncthreads();
    int carry = 0;
    for (int u0 = 0; u0 < n_all; u0 += 1024) {
        const int u = u0 + threadIdx.x;
        int um, t, gold, promote, need = 0;
        if (u < n_all) {
            promote_decide(pv, cs, tau, u, um, t, gold, promote, need);
            if (need && (gold >> pv.logP) >= pv.maxgp) s_err = WGKV_ERR_PT_OVERFLOW;
        }
        int total;
        block_excl_scan(need, s_tmp, &total);
        carry += total;
    }
    __syncthreads();
    if (threadIdx.x == 0 && s_err == 0 && carry > top) s_err = WGKV_ERR_OUT_OF_PAGES;
    __syncthreads();
    if (s_err != 0) {  // block-uniform: leave all state as it was
        if (threadIdx.x == 0) atomicCAS(pv.err_flag, 0, s_err);
        return;
    }
    carry = 0;
    for (int u0 = 0; u0 < n_all; u0 += 1024) {
        const int u = u0 + threadIdx.x;
        int um = 0, t = 0, gold = 0, promote = -1, need = 0;
        if (u < n_all) promote_decide(pv, cs, tau, u, um, t, gold, promote, need);
        int total;
        const int ex = block_excl_scan(need, s_tmp, &total);
        if (u < n_all && promote >= 0) {
            if (need) pv.global_pt[(size_t)um * pv.maxgp + (gold >> pv.logP)] = pv.free_stack[top - 1 - (carry + ex)];
            if (promote) pv.global_len[um] = gold + 1;
            pv.ahead[um] = (t << 1) | promote;
        }
        carry += total;
    }
    if (threadIdx.x == 0) *pv.free_top = top - carry;
}

// The rows of the units that decode_promote_kernel promoted: ring slot t mod W -> global entry G - 1 (G already
// counts the new entry).  Reads everything from the pool's state, so running it again before the layer's decode
// step copies the same row to the same place.
__global__ __launch_bounds__(256) void decode_promote_move_kernel(View pv, CallSeqs cs) {
    const int lpr = pv.row_bytes >> 4;
    const int n_all = cs.n * pv.L * pv.Hkv;
    const int c = blockIdx.x * 256 + threadIdx.x;
    const int u = c / lpr, sub = c % lpr;
    if (u >= n_all) return;
    const int per_layer = cs.n * pv.Hkv;
    const int l = u / per_layer, r = u - l * per_layer;
    const int b = r / pv.Hkv;
    const int sl = cs.sid[b] * pv.L + l;
    const int um = sl * pv.Hkv + r % pv.Hkv;
    const int slot_h = cs.t0[b] % pv.W;
    const int t = pv.seq_len[sl];
    const int ah = pv.ahead[um];
    const int gl = pv.global_len[um];
    int lpage = pv.local_pt[(size_t)um * pv.nlp + (slot_h >> pv.logP)];
    if (ah < 0 || (ah >> 1) != t || !(ah & 1)) return;
    const int slot = t % pv.W;
    if (slot != slot_h) lpage = pv.local_pt[(size_t)um * pv.nlp + (slot >> pv.logP)];
    const int g0 = gl - 1;
    const int gpage = pv.global_pt[(size_t)um * pv.maxgp + (g0 >> pv.logP)];
    const char *rp = page_ptr(pv, lpage) + (size_t)(slot & (pv.P - 1)) * pv.row_bytes + sub * 16;
    const uint4 kk = *reinterpret_cast<const uint4 *>(rp);
    const uint4 vv = *reinterpret_cast<const uint4 *>(rp + pv.v_off);
    char *dp = page_ptr(pv, gpage) + (size_t)(g0 & (pv.P - 1)) * pv.row_bytes + sub * 16;
    *reinterpret_cast<uint4 *>(dp) = kk;
    *reinterpret_cast<uint4 *>(dp + pv.v_off) = vv;
}

// Step (3) of Sec. 4.3 alone, for a call whose units have all been promoted ahead and own their ring pages: one
// round trip (token count, stamp, page of the slot, the new rows) and the stores.  A unit whose stamp does not
// carry the device's token count (a replayed launch whose graph lacks the promotion, a promotion that was
// refused) makes the whole call do nothing and sets the sticky flag.
__global__ __launch_bounds__(1024) void decode_ring_kernel(View pv, CallSeqs cs, DecodeArgs a) {
    __shared__ int s_lpage[kMaxCallUnits];
    __shared__ int s_t[kMaxCallSeqs];
    const int n_units = cs.n * pv.Hkv;
    const int lpr = pv.row_bytes >> 4, n_items = n_units * lpr;
    uint4 kn = make_uint4(0, 0, 0, 0), vn = kn;
    if ((int)threadIdx.x < n_items) {
        const size_t row = (size_t)(threadIdx.x / lpr) * pv.row_bytes + (threadIdx.x % lpr) * 16;
        kn = *reinterpret_cast<const uint4 *>(a.k + row);
        vn = *reinterpret_cast<const uint4 *>(a.v + row);
    }
    const int u = threadIdx.x;
    int bad = 0, mask = 0;
    if (u < n_units) {
        const int b = u / pv.Hkv, h = u % pv.Hkv;
        const int um = unit_meta(pv, cs.sid[b], a.layer, h);
        const int slot_h = cs.t0[b] % pv.W;
        const int t = pv.seq_len[cs.sid[b] * pv.L + a.layer];
        const int ah = pv.ahead[um];
        int lpage = pv.local_pt[(size_t)um * pv.nlp + (slot_h >> pv.logP)];
        const int slot = t % pv.W;
        if (slot != slot_h) lpage = pv.local_pt[(size_t)um * pv.nlp + (slot >> pv.logP)];  // a replayed launch
        bad = ah < 0 || (ah >> 1) != t || lpage < 0;
        s_lpage[u] = lpage;
        if (h == 0) s_t[b] = t;
        mask = ah & 1;
    }
    if (__syncthreads_or(bad)) {  // block-uniform
        if (threadIdx.x == 0) atomicCAS(pv.err_flag, 0, WGKV_ERR_NOT_PROMOTED);
        return;
    }
    if (u < n_units && a.promoted_out) a.promoted_out[u] = (uint8_t)mask;
    if ((int)threadIdx.x < cs.n) pv.seq_len[cs.sid[threadIdx.x] * pv.L + a.layer] = s_t[threadIdx.x] + 1;
    for (int c = threadIdx.x; c < n_items; c += blockDim.x) {
        const int uu = c / lpr, sub = c % lpr;
        const int b = uu / pv.Hkv, h = uu % pv.Hkv;
        const int m = unit_meta(pv, cs.sid[b], a.layer, h);
        const int sl = s_t[b] % pv.W;
        char *rp = page_ptr(pv, s_lpage[uu]) + (size_t)(sl & (pv.P - 1)) * pv.row_bytes + sub * 16;
        if (c != (int)threadIdx.x) {
            const size_t row = (size_t)uu * pv.row_bytes + sub * 16;
            kn = *reinterpret_cast<const uint4 *>(a.k + row);
            vn = *reinterpret_cast<const uint4 *>(a.v + row);
        }
        *reinterpret_cast<uint4 *>(rp) = kn;
        *reinterpret_cast<uint4 *>(rp + pv.v_off) = vn;
        if (sub == 0) pv.ring_g[(size_t)m * pv.W + sl] = a.g[uu];
    }
}

__global__ __launch_bounds__(256) void free_seq_kernel(View pv, int sid) {
    __shared__ int s_tmp[20];
    const int n_units = pv.L * pv.Hkv;
    const int top = *pv.free_top;
    int carry = 0;
    for (int u0 = 0; u0 < n_units; u0 += 256) {
        const int u = u0 + threadIdx.x;
        int n = 0, um = 0, ngp = 0, touched = 0;
        if (u < n_units) {
            um = sid * n_units + u;  // (sid*L + layer)*Hkv + h with u = layer*Hkv + h
            touched = pv.local_pt[(size_t)um * pv.nlp] >= 0;
            ngp = (pv.global_len[um] + pv.P - 1) >> pv.logP;
            n = touched ? pv.nlp + ngp : 0;
        }
        int total;
        const int ex = block_excl_scan(n, s_tmp, &total);
        if (u < n_units) {
            int o = top + carry + ex;
            if (touched) {
                for (int i = 0; i < pv.nlp; i++) {
                    pv.free_stack[o++] = pv.local_pt[(size_t)um * pv.nlp + i];
                    pv.local_pt[(size_t)um * pv.nlp + i] = -1;
                }
                for (int i = 0; i < ngp; i++) {
                    pv.free_stack[o++] = pv.global_pt[(size_t)um * pv.maxgp + i];
                    pv.global_pt[(size_t)um * pv.maxgp + i] = -1;
                }
            }
            pv.global_len[um] = 0;
            pv.ahead[um] = -1;
            for (int s = 0; s < pv.W; s++) pv.ring_g[(size_t)um * pv.W + s] = 0.0f;
        }
        carry += total;
    }
    for (int l = threadIdx.x; l < pv.L; l += 256) pv.seq_len[sid * pv.L + l] = 0;
    __syncthreads();
    if (threadIdx.x == 0) *pv.free_top = top + carry;
}

// A kernel, not a memset: the call may sit in a captured graph.
__global__ void clear_error_kernel(View pv) { *pv.err_flag = 0; }

// ---- host-side launchers (called from the C ABI layer) ----

hipError_t launch_clear_error(const View &pv, hipStream_t st) {
    hipLaunchKernelGGL(clear_error_kernel, dim3(1), dim3(1), 0, st, pv);
    return hipGetLastError();
}

hipError_t launch_init(const View &pv, hipStream_t st) {
    hipLaunchKernelGGL(init_kernel, dim3(4096), dim3(256), 0, st, pv);
    return hipGetLastError();
}

hipError_t launch_prefill(const View &pv, const CallSeqs &cs, int layer, float tau, const void *k,
                          const void *v, const float *g, uint8_t *admit_out, int32_t *cnt,
                          int32_t *plan, int nblk_leave_max, int max_T, int max_empty_ring_rows,
                          int max_admitted, hipStream_t st) {
    PrefillArgs a;
    a.layer = layer;
    a.tau = tau;
    a.k = (const char *)k;
    a.v = (const char *)v;
    a.g = g;
    a.admit_out = admit_out;
    a.cnt = cnt;
    a.plan = plan;
    a.nblk_max = nblk_leave_max > 0 ? nblk_leave_max : 1;
    a.max_adm = max_admitted;
    const int n_units = cs.n * pv.Hkv;
    int gx = a.nblk_max;
    if (admit_out) gx = max(gx, (max_T + kPrefillBlk - 1) / kPrefillBlk);
    hipLaunchKernelGGL(prefill_count_kernel, dim3(gx, n_units), dim3(256), 0, st, pv, cs, a);
    hipLaunchKernelGGL(prefill_plan_kernel, dim3(1), dim3(kPlanThreads), 0, st, pv, cs, a);
    // blocks 0 .. nblk_max-1 of a unit: leaving tokens (and the ring slots they vacate); the rest: ring rows
    // that go to slots still empty (max_empty_ring_rows: the most ring rows of a sequence that has any such)
    const int lpr = pv.row_bytes >> 4;
    const int gxr = (max_empty_ring_rows * lpr + 255) / 256;
    if (nblk_leave_max > 0 || gxr > 0)
        hipLaunchKernelGGL(prefill_scatter_kernel, dim3(a.nblk_max + gxr, n_units), dim3(256), 0, st, pv, cs, a);
    return hipGetLastError();
}

hipError_t launch_decode_step(const View &pv, const CallSeqs &cs, int layer, float tau,
                              const void *k, const void *v, const float *g, uint8_t *promoted_out,
                              hipStream_t st) {
    DecodeArgs a;
    a.layer = layer;
    a.tau = tau;
    a.k = (const char *)k;
    a.v = (const char *)v;
    a.g = g;
    a.promoted_out = promoted_out;
    hipLaunchKernelGGL(decode_step_kernel, dim3(1), dim3(1024), 0, st, pv, cs, a);
    return hipGetLastError();
}

// ring_only: every unit of the call was promoted ahead and owns its ring pages (as far as the host knows; the
// kernel checks)
hipError_t launch_decode_ring(const View &pv, const CallSeqs &cs, int layer, const void *k, const void *v,
                              const float *g, uint8_t *promoted_out, hipStream_t st) {
    DecodeArgs a;
    a.layer = layer;
    a.tau = 0.f;
    a.k = (const char *)k;
    a.v = (const char *)v;
    a.g = g;
    a.promoted_out = promoted_out;
    hipLaunchKernelGGL(decode_ring_kernel, dim3(1), dim3(1024), 0, st, pv, cs, a);
    return hipGetLastError();
}

hipError_t launch_decode_promote(const View &pv, const CallSeqs &cs, float tau, hipStream_t st) {
    hipLaunchKernelGGL(decode_promote_kernel, dim3(1), dim3(1024), 0, st, pv, cs, tau);
    const int lpr = pv.row_bytes >> 4;
    const int64_t items = (int64_t)cs.n * pv.L * pv.Hkv * lpr;
    hipLaunchKernelGGL(decode_promote_move_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0, st, pv, cs);
    return hipGetLastError();
}

hipError_t launch_free_seq(const View &pv, int sid, hipStream_t st) {
    hipLaunchKernelGGL(free_seq_kernel, dim3(1), dim3(256), 0, st, pv, sid);
    return hipGetLastError();
}

}  // namespace wgkv
