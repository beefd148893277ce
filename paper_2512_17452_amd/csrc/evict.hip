// Budgeted eviction on the global cache (appendix "Eviction policy implementation"):
// remove from every head its floor(frac * N) lowest-scored entries, pack the survivors
// to the front in place, give the emptied pages back.
//
//  evict_compact_kernel   one block per (sequence, kv head): radix select of the cut in
//                         the total order of the fp32 bit patterns (equal scores: the
//                         older entry goes first), then in-place compaction of K/V rows
//  evict_release_kernel   one block: emptied pages back on the free stack, units in
//                         (position in the call, kv head) order, a unit's pages in
//                         ascending table index
#include "wgkv_dev.h"

namespace wgkv {

constexpr int kEvictThreads = 1024;

struct EvictArgs {
    int layer;
    float frac;
    const float *scores;   // [n_units][stride]
    long long stride;
    int32_t *n_evicted;    // optional [n_units]
    int32_t *released;     // workspace [n_units]: pages each unit gives back
};

__device__ __forceinline__ uint32_t evict_key(float x) {
    const uint32_t u = __float_as_uint(x);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(kEvictThreads) void evict_compact_kernel(View pv, CallSeqs cs, EvictArgs a) {
    __shared__ unsigned s_hist[256];
    __shared__ unsigned s_sel[4];      // prefix, mask, remaining rank
    __shared__ int s_tmp[20];
    __shared__ int s_src[kEvictThreads], s_dst[kEvictThreads];
    const int u = blockIdx.x, b = u / pv.Hkv, h = u % pv.Hkv;
    const int um = unit_meta(pv, cs.sid[b], a.layer, h);
    const int N = pv.global_len[um];
    // a cache longer than the caller's score row (the host's bound was stale): the head is left alone
    const int n_e = N <= a.stride ? (int)floor((double)a.frac * (double)N) : 0;
    if (threadIdx.x == 0) {
        if (a.n_evicted) a.n_evicted[u] = n_e;
        if (n_e == 0) a.released[u] = 0;
    }
    if (n_e == 0) return;  // block-uniform
    const float *sc = a.scores + (size_t)u * a.stride;

    // ---- the n_e-th smallest key: four passes over one byte each, most significant first ----
    if (threadIdx.x == 0) { s_sel[0] = 0u; s_sel[1] = 0u; s_sel[2] = (unsigned)n_e; }
    for (int pass = 3; pass >= 0; pass--) {
        if (threadIdx.x < 256) s_hist[threadIdx.x] = 0u;
        __syncthreads();
        const unsigned prefix = s_sel[0], mask = s_sel[1];
        for (int j = threadIdx.x; j < N; j += kEvictThreads) {
            const uint32_t key = evict_key(sc[j]);
            if ((key & mask) == prefix) atomicAdd(&s_hist[(key >> (8 * pass)) & 255u], 1u);
        }
        __syncthreads();
        // the bin in which the running count reaches the rank: a block-wide prefix over the 256 bins
        {
            const unsigned want = s_sel[2];
            const int cnt = threadIdx.x < 256 ? (int)s_hist[threadIdx.x] : 0;
            int total;
            const int ex = block_excl_scan(cnt, s_tmp, &total);
            __syncthreads();  // everybody has read s_sel
            if (threadIdx.x < 256 && (unsigned)ex < want && want <= (unsigned)(ex + cnt)) {
                s_sel[0] = prefix | ((unsigned)threadIdx.x << (8 * pass));
                s_sel[1] = mask | (255u << (8 * pass));
                s_sel[2] = want - (unsigned)ex;  // rank among the keys that share the longer prefix
            }
        }
        __syncthreads();
    }
    const uint32_t cut = s_sel[0];          // key of the last entry to go
    const int ties_to_go = (int)s_sel[2];   // entries with exactly that key that go (the oldest ones)

    // ---- in-place compaction, tiles of 1024 entries in ascending order ----
    // A survivor moves to an index not above its own, and rows are taken in ascending order with all
    // reads of a group of rows finished before its writes start, so no unread row is overwritten.
    const int cpr = (int)(pv.row_bytes / 16);        // 16-byte chunks per row
    const int rows_per_pass = kEvictThreads / cpr;
    const int my_row = threadIdx.x / cpr, my_chunk = threadIdx.x % cpr;
    const int32_t *gpt = pv.global_pt + (size_t)um * pv.maxgp;
    int ties_seen = 0, kept = 0;
    for (int j0 = 0; j0 < N; j0 += kEvictThreads) {
        const int j = j0 + threadIdx.x;
        uint32_t key = 0xffffffffu;
        if (j < N) key = evict_key(sc[j]);
        const int is_tie = (j < N && key == cut) ? 1 : 0;
        int n_ties;
        const int tie_rank = ties_seen + block_excl_scan(is_tie, s_tmp, &n_ties);
        const int stays = (j < N && !(key < cut || (is_tie && tie_rank < ties_to_go))) ? 1 : 0;
        int n_stay;
        const int idx = block_excl_scan(stays, s_tmp, &n_stay);
        __syncthreads();  // the previous tile's copy loop is done with s_src / s_dst
        if (stays) { s_src[idx] = j; s_dst[idx] = kept + idx; }
        __syncthreads();
        for (int r0 = 0; r0 < n_stay; r0 += rows_per_pass) {
            const int r = r0 + my_row;
            const bool act = my_row < rows_per_pass && r < n_stay && s_src[r] != s_dst[r];
            uint4 kv[2];
            if (act) {
                const int src = s_src[r];
                const char *p = page_ptr(pv, gpt[src >> pv.logP]) + (size_t)(src & (pv.P - 1)) * pv.row_bytes + my_chunk * 16;
                kv[0] = *reinterpret_cast<const uint4 *>(p);
                kv[1] = *reinterpret_cast<const uint4 *>(p + pv.v_off);
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the rows are in registers before anybody writes
            __syncthreads();
            if (act) {
                const int dst = s_dst[r];
                char *p = page_ptr(pv, gpt[dst >> pv.logP]) + (size_t)(dst & (pv.P - 1)) * pv.row_bytes + my_chunk * 16;
                *reinterpret_cast<uint4 *>(p) = kv[0];
                *reinterpret_cast<uint4 *>(p + pv.v_off) = kv[1];
            }
        }
        ties_seen += n_ties;
        kept += n_stay;
    }
    if (threadIdx.x == 0) {
        pv.global_len[um] = kept;  // = N - n_e
        a.released[u] = ((N + pv.P - 1) >> pv.logP) - ((kept + pv.P - 1) >> pv.logP);
    }
}

// global_len already holds the new lengths; released[u] says how many table entries behind the
// last one in use each unit gives back.
__global__ __launch_bounds__(kEvictThreads) void evict_release_kernel(View pv, CallSeqs cs, EvictArgs a, int n_units) {
    __shared__ int s_tmp[20];
    const int u = threadIdx.x;
    int n = 0;
    if (u < n_units) n = a.released[u];
    int total;
    const int ex = block_excl_scan(n, s_tmp, &total);
    const int top = *pv.free_top;
    if (u < n_units && n > 0) {
        const int um = unit_meta(pv, cs.sid[u / pv.Hkv], a.layer, u % pv.Hkv);
        const int first = (pv.global_len[um] + pv.P - 1) >> pv.logP;
        int32_t *gpt = pv.global_pt + (size_t)um * pv.maxgp;
        for (int i = 0; i < n; i++) {
            pv.free_stack[top + ex + i] = gpt[first + i];
            gpt[first + i] = -1;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) *pv.free_top = top + total;
}

size_t evict_ws_bytes(int n_units) { return (size_t)((n_units * 4 + 255) / 256) * 256; }

hipError_t launch_evict_apply(const View &pv, const CallSeqs &cs, int layer, const float *scores,
                              int64_t stride, float frac, int32_t *n_evicted, void *ws, hipStream_t st) {
    const int n_units = cs.n * pv.Hkv;
    if (pv.row_bytes % 16 != 0 || pv.row_bytes / 16 > kEvictThreads) return hipErrorNotSupported;
    EvictArgs a;
    a.layer = layer;
    a.frac = frac;
    a.scores = scores;
    a.stride = stride;
    a.n_evicted = n_evicted;
    a.released = (int32_t *)ws;
    hipLaunchKernelGGL(evict_compact_kernel, dim3(n_units), dim3(kEvictThreads), 0, st, pv, cs, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(evict_release_kernel, dim3(1), dim3(kEvictThreads), 0, st, pv, cs, a, n_units);
    return hipGetLastError();
}

}  // namespace wgkv
