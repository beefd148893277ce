// Device-side view of the pool and small helpers shared by the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/wgkv.h"

namespace wgkv {

constexpr int kMaxCallSeqs = WGKV_MAX_CALL_SEQS;
constexpr int kMaxCallUnits = WGKV_MAX_CALL_UNITS;

// Everything a kernel needs to find its way through pool and metadata.
struct View {
    int32_t L, Hq, Hkv, d, dtype, es;   // es: bytes per element
    int32_t P, logP, W, S, maxgp, nlp;  // nlp = ceil(W/P) local pages per head
    int32_t G;                           // query heads per kv head
    int32_t n_pages;
    uint32_t row_bytes;                  // d * es
    uint32_t v_off;                      // byte offset of the V half of a page: P * d * es
    uint64_t page_bytes;                 // 2 * P * d * es
    char *pool;
    int32_t *seq_len, *global_len, *local_pt, *global_pt;
    float *ring_g;
    int32_t *free_stack, *free_top, *err_flag;
    int32_t *unit_counters;              // [kMaxCallUnits], zero between calls
    int32_t *ahead;                      // [S][L][Hkv]: (t << 1) | promoted once the promotion of the step that
                                         // feeds token t has been done ahead of its ring write, else -1
};

// The sequences of one call, passed by value in the kernel arguments.
struct CallSeqs {
    int32_t n;
    int32_t sid[kMaxCallSeqs];   // sequence slot
    int32_t t0[kMaxCallSeqs];    // tokens seen before this call (host mirror of seq_len)
    int32_t ntok[kMaxCallSeqs];  // tokens / queries of this call
    int32_t base[kMaxCallSeqs];  // first packed row of the sequence
};

__device__ __forceinline__ int unit_meta(const View &pv, int sid, int layer, int h) {
    return (sid * pv.L + layer) * pv.Hkv + h;
}

__device__ __forceinline__ char *page_ptr(const View &pv, int page) {
    return pv.pool + (uint64_t)(uint32_t)page * pv.page_bytes;
}

// Work items (x, head, z) of a 1-D launch of nx * nh * nz blocks.  Blocks go to the 8 XCDs
// round-robin by their index, and each XCD has its own L2: when the heads divide evenly, an XCD
// gets all blocks of its heads and of no others, so the blocks that stream the same K/V (or Q/dO)
// tiles of a head share one L2 instead of pulling eight copies through eight of them.  Inside an
// XCD the order is z, head, x ascending (callers put the heaviest x first).
__device__ __forceinline__ void xcd_item(int nx, int nh, int nz, int &x, int &h, int &z) {
    constexpr int kXcds = 8;
    const int n = (int)blockIdx.x;
    (void)nz;
    if (nh % kXcds == 0) {
        const int xcd = n % kXcds, r = n / kXcds, hpx = nh / kXcds;
        z = r / (hpx * nx);
        const int rem = r - z * hpx * nx;
        h = xcd + kXcds * (rem / nx);
        x = rem % nx;
    } else {
        x = n % nx;
        h = (n / nx) % nh;
        z = n / (nx * nh);
    }
}

// 16 bytes that are read once per launch and have left every cache before anybody reads them
// again (K/V rows in decode attention, hidden rows in the linear gate, rows that admission
// copies): a load with the non-temporal hint.  On this machine such loads stream 8-10 % faster
// than plain ones (a read-only kernel: 6.9 against 6.2 TB/s); tiles that many blocks share
// are read with plain loads.
typedef unsigned wg_u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_once16(const char *p) {
    const wg_u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const wg_u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// ---- wave64 cross-lane helpers (DPP where the pattern allows) ----

template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ int dpp_i(int x) {
    return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xf, 0xf, true);
}

constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside each 8 lanes
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i inside each 16 lanes
constexpr int kDppShl4 = 0x104;       // lane i reads lane i+4 of its row of 16
constexpr int kDppShr4 = 0x114;       // lane i reads lane i-4
constexpr int kDppRor4 = 0x124;       // rotate the row of 16 by 4
constexpr int kDppRor8 = 0x128;       // rotate by 8: lane i <-> i^8

// v_permlane32_swap / v_permlane16_swap exchange halves (quarters) of two registers
// inside the vector unit, without the LDS crossbar that ds_bpermute goes through.
// swap32(a, b): lanes 0-31 get (a[l], a[l+32]), lanes 32-63 get (b[l-32], b[l]);
// swap16(a, b): rows 0 and 2 of 16 lanes get (a[l], a[l+16]), rows 1 and 3 get (b[l-16], b[l]).
// With a == b every lane holds its own value and that of lane l^32 (l^16); with two
// different values, adding the pair halves two partial sums into one per lane.
struct LanePair {
    float a, b;
};
// (Written as assembly: with the compiler builtins of this toolchain, arithmetic on the
// two results reads the first one twice.  The s_nop covers the wait states the
// instruction needs after a vector write of its operands.)
__device__ __forceinline__ LanePair swap32(float a, float b) {
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return {a, b};
}
__device__ __forceinline__ LanePair swap16(float a, float b) {
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
    return {a, b};
}
// The value of lane l ^ OFF (OFF = 8, 16 or 32), again without the LDS crossbar.
template <int OFF>
__device__ __forceinline__ float lane_xor(float x, int lane) {
    static_assert(OFF == 8 || OFF == 16 || OFF == 32, "");
    if constexpr (OFF == 8) {
        return dpp_f<0x128>(x);  // rotate the row of 16 by 8
    } else if constexpr (OFF == 16) {
        const LanePair r = swap16(x, x);
        return (lane & 16) ? r.a : r.b;
    } else {
        const LanePair r = swap32(x, x);
        return (lane & 32) ? r.a : r.b;
    }
}
__device__ __forceinline__ float sum_xor32(float x) { const LanePair r = swap32(x, x); return r.a + r.b; }
__device__ __forceinline__ float sum_xor16(float x) { const LanePair r = swap16(x, x); return r.a + r.b; }
__device__ __forceinline__ float max_xor32(float x) { const LanePair r = swap32(x, x); return fmaxf(r.a, r.b); }

// Sum over aligned groups of N consecutive lanes; every lane of the group gets the total.
template <int N>
__device__ __forceinline__ float group_sum(float x) {
    static_assert(N == 1 || N == 2 || N == 4 || N == 8 || N == 16 || N == 32 || N == 64, "");
    if (N >= 2) x += dpp_f<kDppXor1>(x);
    if (N >= 4) x += dpp_f<kDppXor2>(x);
    if (N >= 8) x += dpp_f<kDppHalfMirror>(x);
    if (N >= 16) x += dpp_f<kDppMirror>(x);
    if (N >= 32) x = sum_xor16(x);
    if (N >= 64) x = sum_xor32(x);
    return x;
}

// Inclusive prefix over the 64 lanes, in the vector unit (DPP) instead of six trips through the
// LDS crossbar: sums of 4 from the original values (row_shr 1, 2, 3; lanes shifted in from
// outside a row of 16 read zero), then of 8 and 16 inside the row, then lane 15 of the row before
// into rows 1 and 3 (row_bcast15) and lane 31 into rows 2 and 3 (row_bcast31).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_masked_i(int x) {
    return __builtin_amdgcn_update_dpp(0, x, CTRL, ROW_MASK, 0xf, true);
}
__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
    (void)lane;
    int t = v + dpp_masked_i<0x111, 0xf>(v);
    t += dpp_masked_i<0x112, 0xf>(v);
    t += dpp_masked_i<0x113, 0xf>(v);
    t += dpp_masked_i<0x114, 0xf>(t);
    t += dpp_masked_i<0x118, 0xf>(t);
    t += dpp_masked_i<0x142, 0xa>(t);
    t += dpp_masked_i<0x143, 0xc>(t);
    return t;
}

// Exclusive prefix over the values of one block of up to 1024 threads.  s_tmp: >= 16 ints.
// Returns the exclusive prefix of v for this thread; *total gets the block sum.  Every thread adds
// up the totals of the waves before its own by itself (at most 16 values, read as a broadcast),
// so there is no serial pass of one thread and only the two barriers around the hand-over.
__device__ __forceinline__ int block_excl_scan(int v, int *s_tmp, int *total) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    const int inc = wave_incl_scan(v, lane);
    __syncthreads();  // s_tmp may still be read from an earlier call
    if (lane == 63) s_tmp[w] = inc;
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int i = 0; i < 16; i++) {
        const int x = i < nw ? s_tmp[i] : 0;
        before += i < w ? x : 0;
        all += x;
    }
    *total = all;
    return inc - v + before;
}

}  // namespace wgkv
