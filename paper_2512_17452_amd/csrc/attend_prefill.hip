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
// K and V tiles are staged row-major; the V^T operand is read from the V tile with the
// transposing LDS load.  Everything is computed transposed, S^T = K Q^T and O^T = V^T P^T with
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
constexpr int kPfKStride = 272;   // bytes per key row of the K tile in LDS (256 + 16 pad): rows are read whole
constexpr int kPfVStride = 320;   // bytes per key row of the V tile (256 + 64 pad): columns are read, four
                                  // rows and 64 bytes of each at a time per half wave, which this stride
                                  // spreads over all banks

struct PrefillAttnArgs {
    int nx;                 // blocks per (sequence, kv head) of the launch
    const int32_t *order;   // [n_units] (sequence, kv head) units, the one with the longest global cache first
    int layer;
    float tau;
    float scale_log2e;
    const char *q, *k, *v;  // chunk tensors, bf16
    const float *g;         // chunk scores
    float *out;
};

// A operand of O^T += V^T P^T from the row-major V tile: the output row of this lane is
// d = db*32 + qn, its 8 contraction slots are keys r0 + 4*half + {0..3} and r0 + 8 + 4*half + {0..3}
// of the tile.  ds_read_b64_tr_b16 transposes inside groups of 16 lanes: lane i of a group receives
// element i%4 of the 8 bytes addressed by lanes i/4, 4 + i/4, 8 + i/4 and 12 + i/4, so lane s of a
// group addresses (key s/4 of the four, columns 4*(s%4)..+3 of the group's 16).
typedef short pf_s16x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ pf_bf16x8_t pf_get_cols(const char *tile, int lane, int db, int r0) {
    const int half = lane >> 5;
    const char *p = tile + (r0 + 4 * half + ((lane & 15) >> 2)) * kPfVStride +
                    (db * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
    typedef pf_s16x4_t __attribute__((address_space(3))) *lds_ptr_t;
    const pf_s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)p);
    const pf_s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 8 * kPfVStride));
    const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
    const uint4 u4 = make_uint4(l2.x, l2.y, h2.x, h2.y);
    return __builtin_bit_cast(pf_bf16x8_t, u4);
}

__device__ __forceinline__ uint32_t pf_pack(float lo, float hi) {
    pf_bf16x2_t t = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, t);
}

__global__ __launch_bounds__(512) void attend_prefill_kernel(View pv, CallSeqs cs, PrefillAttnArgs a) {
    __shared__ __attribute__((aligned(16))) char s_k[2][kPfKT * kPfKStride];
    __shared__ __attribute__((aligned(16))) char s_v[2][kPfKT * kPfVStride];
    __shared__ __attribute__((aligned(16))) int s_lo[2][kPfKT];
    __shared__ __attribute__((aligned(16))) int s_hi[2][kPfKT];

    // Blocks are handed out in the order of their index and go to the 8 XCDs round-robin: all
    // blocks of the unit with the longest global cache come first, its latest positions (which see
    // the most chunk keys) at the front, then the next unit.  Admission is head-specific, so units
    // differ several-fold in work: with the long ones at the front the launch does not end on a
    // late-started long one, and every unit is spread evenly over the XCDs (giving each XCD whole
    // heads, for the sake of its L2, leaves the XCDs as unbalanced as the heads are).
    const int unit = a.order[blockIdx.x / a.nx];
    const int b = unit / pv.Hkv, h = unit % pv.Hkv;
    const int qt = a.nx - 1 - (int)(blockIdx.x % a.nx);
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

    // ---- staging of a key tile: thread -> (key of the tile, 16-byte d chunk), K and V row-major ----
    const int ld_key = threadIdx.x >> 4, ld_dc = threadIdx.x & 15;
    // two sets of staging registers: a tile is requested two iterations before it is multiplied
    // (plain variables passed one by one: a struct of them ends up in scratch memory)
    uint4 k0r, v0r, k1r, v1r;
    int lo0r, hi0r, lo1r, hi1r;
    // Page ids live in registers, one per lane, so that the address of a key row never
    // waits for a page-table load: 64 consecutive entries of the global table (reloaded
    // every 64 pages) and the whole local table when it has at most 64 entries.
    int pt_base = 0;
    int ptreg = (lane < pv.maxgp) ? pv.global_pt[(size_t)um * pv.maxgp + lane] : 0;
    const bool lp_in_reg = pv.nlp <= 64;
    const int lpreg = (lp_in_reg && lane < pv.nlp) ? pv.local_pt[(size_t)um * pv.nlp + lane] : 0;
    const int slot0 = t0 > pv.W ? t0 % pv.W : 0;  // ring slot of the oldest position
    const int64_t v_delta_chunk = a.v - a.k;
    auto fetch = [&](int t, uint4 &r_k, uint4 &r_v, int &r_lo, int &r_hi) __attribute__((always_inline)) {
        const char *kp;
        int64_t v_delta;
        int lo = INT_MAX, hi = INT_MAX;  // invisible unless shown otherwise
        if (t < n_g) {  // global cache: visible to every query
            if (((t * kPfKT + kPfKT - 1) >> pv.logP) >= pt_base + 64) {
                pt_base = (t * kPfKT) >> pv.logP;
                ptreg = (pt_base + lane < pv.maxgp) ? pv.global_pt[(size_t)um * pv.maxgp + pt_base + lane] : 0;
            }
            const int idx = t * kPfKT + ld_key, idc = min(idx, gl - 1);
            const int pg = __shfl(ptreg, (idc >> pv.logP) - pt_base);
            kp = page_ptr(pv, pg) + (size_t)(idc & (pv.P - 1)) * (kPfD * 2);
            if (idx < gl) lo = INT_MIN;
            v_delta = pv.v_off;
        } else if (t < n_g + n_r) {  // ring, oldest position first
            const int idx = (t - n_g) * kPfKT + ld_key, idc = min(idx, w_eff - 1);
            int slot = slot0 + idc;
            slot = slot >= pv.W ? slot - pv.W : slot;
            const int pos = t0 - w_eff + idc;
            const int pg = lp_in_reg ? __shfl(lpreg, slot >> pv.logP)
                                     : pv.local_pt[(size_t)um * pv.nlp + (slot >> pv.logP)];
            kp = page_ptr(pv, pg) + (size_t)(slot & (pv.P - 1)) * (kPfD * 2);
            if (idx < w_eff) {
                lo = pos;
                hi = (pv.ring_g[(size_t)um * pv.W + slot] >= a.tau) ? INT_MAX : pos + pv.W - 1;
            }
            v_delta = pv.v_off;
        } else {  // this chunk
            const int idx = (t - n_g - n_r) * kPfKT + ld_key, idc = min(idx, T - 1);
            const size_t row = (size_t)(base + idc) * pv.Hkv + h;
            kp = a.k + row * (kPfD * 2);
            if (idx < T) {
                lo = t0 + idx;
                hi = (a.g[row] >= a.tau) ? INT_MAX : t0 + idx + pv.W - 1;
            }
            v_delta = v_delta_chunk;
        }
        r_k = *reinterpret_cast<const uint4 *>(kp + ld_dc * 16);
        r_v = *reinterpret_cast<const uint4 *>(kp + v_delta + ld_dc * 16);
        r_lo = lo;
        r_hi = hi;
    };
    // Full tiles of the global cache, pages of at least 4 tokens: the four keys a wave
    // stages share a page, so the page base is scalar and a lane only adds a fixed offset.
    const bool lean_ok = pv.P >= 4;
    const uint32_t lean_k_off = (uint32_t)(ld_key & (pv.P - 1)) * (kPfD * 2) + ld_dc * 16;
    auto fetch_lean = [&](int t, uint4 &r_k, uint4 &r_v, int &r_lo, int &r_hi) __attribute__((always_inline)) {
        if (((t * kPfKT + kPfKT - 1) >> pv.logP) >= pt_base + 64) {
            pt_base = (t * kPfKT) >> pv.logP;
            ptreg = (pt_base + lane < pv.maxgp) ? pv.global_pt[(size_t)um * pv.maxgp + pt_base + lane] : 0;
        }
        const int pg = __builtin_amdgcn_readlane(ptreg, ((t * kPfKT + 4 * wave) >> pv.logP) - pt_base);
        // inside its page the tile begins at row (32 t) mod P (0 unless a page holds several tiles)
        const char *sb = page_ptr(pv, pg) + (size_t)((t * kPfKT) & (pv.P - 1)) * (kPfD * 2);
        r_k = *reinterpret_cast<const uint4 *>(sb + lean_k_off);
        r_v = *reinterpret_cast<const uint4 *>(sb + lean_k_off + pv.v_off);
        r_lo = INT_MIN;
        r_hi = INT_MAX;
    };
    auto stage = [&](int buf, const uint4 &r_k, const uint4 &r_v, int r_lo, int r_hi) __attribute__((always_inline)) {
        *reinterpret_cast<uint4 *>(&s_k[buf][ld_key * kPfKStride + ld_dc * 16]) = r_k;
        *reinterpret_cast<uint4 *>(&s_v[buf][ld_key * kPfVStride + ld_dc * 16]) = r_v;
        if (ld_dc == 0) { s_lo[buf][ld_key] = r_lo; s_hi[buf][ld_key] = r_hi; }
    };

    const int n_plain = gl / kPfKT;  // full tiles of the global cache: no mask
    auto fetch_any = [&](int t, uint4 &r_k, uint4 &r_v, int &r_lo, int &r_hi) __attribute__((always_inline)) {
        if (lean_ok && t < n_plain) fetch_lean(t, r_k, r_v, r_lo, r_hi);
        else fetch(t, r_k, r_v, r_lo, r_hi);
    };
    fetch_any(0, k0r, v0r, lo0r, hi0r);
    stage(0, k0r, v0r, lo0r, hi0r);
    if (n_tiles > 1) fetch_any(1, k1r, v1r, lo1r, hi1r);
    __syncthreads();

    // one iteration: tile t is multiplied, tile t+2 is requested into rf, tile t+1 goes from rs to LDS
    auto body = [&](int t, uint4 &f_k, uint4 &f_v, int &f_lo, int &f_hi, const uint4 &s_kk, const uint4 &s_vv,
                    const int &s_lo_, const int &s_hi_) __attribute__((always_inline)) {
        const int buf = t & 1;
        // LDS latency is the scarce thing here: the eight K fragments are requested at once,
        // the address arithmetic and global loads of the next tile run while they arrive,
        // and the V fragments are requested before the softmax that hides their latency.
        pf_bf16x8_t ka[8];
#pragma unroll
        for (int ks = 0; ks < 8; ks++)
            ka[ks] = *reinterpret_cast<const pf_bf16x8_t *>(&s_k[buf][qn * kPfKStride + (ks * 16 + half * 8) * 2]);
        __builtin_amdgcn_sched_barrier(0);
        if (t + 2 < n_tiles) fetch_any(t + 2, f_k, f_v, f_lo, f_hi);  // in flight while this tile and the next are multiplied
        __builtin_amdgcn_sched_barrier(0);

        // ---- S^T = K Q^T : rows = keys of the tile, columns = this wave's queries ----
        pf_f32x16_t s;
#pragma unroll
        for (int c = 0; c < 16; c++) s[c] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ks++) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qv[ks], s, 0, 0, 0);
        // V^T fragments read column-wise from the row-major V tile
        pf_bf16x8_t va[2][4];
#pragma unroll
        for (int t2 = 0; t2 < 2; t2++)
#pragma unroll
            for (int db = 0; db < 4; db++) va[t2][db] = pf_get_cols(s_v[buf], lane, db, 16 * t2);
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
        if (t + 1 < n_tiles) stage(buf ^ 1, s_kk, s_vv, s_lo_, s_hi_);
        __syncthreads();
    };
    {
        int t = 0;
        for (; t + 1 < n_tiles; t += 2) {
            body(t, k0r, v0r, lo0r, hi0r, k1r, v1r, lo1r, hi1r);
            body(t + 1, k1r, v1r, lo1r, hi1r, k0r, v0r, lo0r, hi0r);
        }
        if (t < n_tiles) body(t, k0r, v0r, lo0r, hi0r, k1r, v1r, lo1r, hi1r);
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

// Units of the call by descending length of their global cache (equal lengths: lower unit first).
__global__ __launch_bounds__(1024) void prefill_order_kernel(View pv, CallSeqs cs, int layer, int32_t *order) {
    __shared__ int s_len[kMaxCallUnits];
    const int n_units = cs.n * pv.Hkv, u = threadIdx.x;
    if (u < n_units) s_len[u] = pv.global_len[unit_meta(pv, cs.sid[u / pv.Hkv], layer, u % pv.Hkv)];
    __syncthreads();
    if (u < n_units) {
        const int mine = s_len[u];
        int rank = 0;
        for (int v = 0; v < n_units; v++) rank += (s_len[v] > mine || (s_len[v] == mine && v < u)) ? 1 : 0;
        order[rank] = u;
    }
}

size_t attend_prefill_ws_bytes(const View &pv, int n_seqs, int64_t total_q) {
    (void)pv; (void)n_seqs; (void)total_q;
    return 256 + sizeof(int32_t) * kMaxCallUnits;  // the order of the units; everything else stays in registers and LDS
}

hipError_t launch_attend_prefill(const View &pv, const CallSeqs &cs, int layer, const void *q,
                                 const void *k, const void *v, const float *g, float tau,
                                 float scale, float *out, void *ws, hipStream_t st) {
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
    a.nx = (max_t + kPfQ - 1) / kPfQ;
    a.order = (const int32_t *)ws;
    hipLaunchKernelGGL(prefill_order_kernel, dim3(1), dim3(1024), 0, st, pv, cs, layer, (int32_t *)ws);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(attend_prefill_kernel, dim3(a.nx * pv.Hkv * cs.n), dim3(512), 0, st, pv, cs, a);
    return hipGetLastError();
}

}  // namespace wgkv
