// Per-head line selection (Alg. 2 from Desc_Sort on) and top-B retention (Alg. 3), gfx950.
//
//   sort_kernel   one workgroup per (head, list): stable LSD radix sort (4 x 8 bits) of the n line
//                 weights in descending order; equal weights keep ascending index order.  Each of
//                 the 16 waves owns a contiguous slice of the input, counts its digits in its own
//                 LDS histogram, and scatters its slice in order: inside a 64-element chunk the
//                 rank among equal digits comes from wave ballots, across chunks from the wave's
//                 running counters.  No atomics decide an output position.
//   walk_kernel   one workgroup per head: the sequential greedy loop of Alg. 2, run by one lane in
//                 binary32 with the operation order of the definition; the sorted lists are
//                 streamed through LDS in chunks by the whole workgroup.
//   emit_kernel   one workgroup per (head, list): the chosen prefix of a sorted list becomes an
//                 ascending index list (bitmap in LDS + prefix popcount).
//   topb_kernel   Alg. 3: the `budget` largest scores per KV head by 4-pass radix select on the
//                 float bit patterns, ties broken towards smaller indices, ascending output.
#include "ls_device.h"
#include "ls_internal.h"

namespace ls {

// order-preserving map float -> uint32 (ascending), then inverted so ascending keys = descending floats
__device__ __forceinline__ uint32_t desc_key(float x) {
    const uint32_t u = __builtin_bit_cast(uint32_t, x);
    const uint32_t asc = u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
    return ~asc;
}
__device__ __forceinline__ float key_to_float(uint32_t key) {
    const uint32_t asc = ~key;
    const uint32_t u = (asc >> 31) ? (asc ^ 0x80000000u) : ~asc;
    return __builtin_bit_cast(float, u);
}

constexpr int SORT_THREADS = 1024;
constexpr int SORT_WAVES = 16;

// grid (2, BH): list 0 = diagonals (slash), 1 = columns (vert).
__global__ __launch_bounds__(SORT_THREADS) void sort_kernel(SelectArgs a) {
    __shared__ uint32_t hist[SORT_WAVES][256];
    __shared__ uint32_t dbase[256];
    const int list = blockIdx.x, bh = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int64_t n = a.n;
    const float* src = (list == 0 ? a.slash : a.vert) + (int64_t)bh * n;
    const int64_t seg = ((int64_t)list * a.BH + bh) * n;
    uint32_t* kbuf[2] = {a.skey0 + seg, a.skey1 + seg};
    int32_t* ibuf[2] = {a.sidx0 + seg, a.sidx1 + seg};
    const int64_t slice = (((n + SORT_WAVES - 1) / SORT_WAVES) + 63) / 64 * 64;
    const int64_t lo = (int64_t)wv * slice;
    const int64_t hi = lo + slice < n ? lo + slice : n;

    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 8 * pass;
        const uint32_t* kin = kbuf[(pass + 1) & 1];        // pass 0 reads src directly
        const int32_t* iin = ibuf[(pass + 1) & 1];
        uint32_t* kout = kbuf[pass & 1];
        int32_t* iout = ibuf[pass & 1];
        for (int i = tid; i < SORT_WAVES * 256; i += SORT_THREADS) (&hist[0][0])[i] = 0u;
        __syncthreads();
        for (int64_t i = lo + lane; i < hi; i += 64) {
            const uint32_t key = pass == 0 ? desc_key(src[i]) : kin[i];
            atomicAdd(&hist[wv][(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        // exclusive offsets in (digit, wave) order
        if (tid < 256) {
            uint32_t run = 0;
            for (int w = 0; w < SORT_WAVES; ++w) { const uint32_t t = hist[w][tid]; hist[w][tid] = run; run += t; }
            dbase[tid] = run;
        }
        __syncthreads();
        if (tid < 64) {                                    // scan of 256 digit totals by one wave
            uint32_t v[4], s = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) { v[q] = dbase[4 * tid + q]; s += v[q]; }
            uint32_t inc = s;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) { const uint32_t t = __shfl_up(inc, off, 64); if (lane >= off) inc += t; }
            uint32_t ex = inc - s;
#pragma unroll
            for (int q = 0; q < 4; ++q) { dbase[4 * tid + q] = ex; ex += v[q]; }
        }
        __syncthreads();
        if (tid < 256) {
            const uint32_t bs = dbase[tid];
            for (int w = 0; w < SORT_WAVES; ++w) hist[w][tid] += bs;
        }
        __syncthreads();
        // in-order scatter of this wave's slice
        volatile uint32_t* myh = hist[wv];
        for (int64_t c0 = lo; c0 < hi; c0 += 64) {
            const int64_t i = c0 + lane;
            const bool ok = i < hi;
            uint32_t key = 0; int32_t idx = 0;
            if (ok) { key = pass == 0 ? desc_key(src[i]) : kin[i]; idx = pass == 0 ? (int32_t)i : iin[i]; }
            const uint32_t dg = (key >> shift) & 255u;
            uint64_t peers = __ballot(ok);
#pragma unroll
            for (int bit = 0; bit < 8; ++bit) {
                const bool one = (dg >> bit) & 1u;
                const uint64_t bal = __ballot(ok && one);
                peers &= one ? bal : ~bal;
            }
            const uint64_t below = peers & ((1ull << lane) - 1ull);
            const uint32_t rank = __popcll(below);
            uint32_t base = 0;
            if (ok) base = myh[dg];
            __builtin_amdgcn_wave_barrier();
            if (ok) {
                kout[base + rank] = key;
                iout[base + rank] = idx;
                if (below == 0ull) myh[dg] = base + (uint32_t)__popcll(peers);
            }
            __builtin_amdgcn_wave_barrier();
        }
        __threadfence_block();
        __syncthreads();
    }
    // after 4 passes the result sits in buffer 1 ((3 & 1) = 1); attach weight and the line's largest entry
    const uint32_t* kfin = kbuf[1];
    const int32_t* ifin = ibuf[1];
    const float* mx = (list == 0 ? a.smax : a.vmax) + (int64_t)bh * n;
    float* ow = a.sorted_w + seg;
    float* om = a.sorted_m + seg;
    for (int64_t i = tid; i < n; i += SORT_THREADS) {
        ow[i] = key_to_float(kfin[i]);
        om[i] = mx[ifin[i]];
    }
}

// ---- the greedy loop ----------------------------------------------------------------------------
constexpr int WALK_THREADS = 256;
constexpr int WALK_CHUNK = 2048;

struct WalkState { int is, iv; float ol_s, ol_v, sum; int done; };

// grid (BH).  Reads the sorted lists (weights, maxima, indices) and writes taken counts.
// The whole workgroup copies a window of each list (starting at that list's head) into LDS; lane 0
// then walks while both heads and their successors are inside the windows.  The walking lane keeps
// the two heads and their successors in registers, so an LDS read is issued one step before its
// value is needed.
__global__ __launch_bounds__(WALK_THREADS) void walk_kernel(SelectArgs a) {
    __shared__ float cw[2][WALK_CHUNK], cm[2][WALK_CHUNK], cl[2][WALK_CHUNK];
    __shared__ WalkState st;
    const int bh = blockIdx.x, tid = threadIdx.x;
    const int n = (int)a.n;
    const int64_t nh = a.n_hat;
    const int64_t seg_s = ((int64_t)0 * a.BH + bh) * a.n, seg_v = ((int64_t)1 * a.BH + bh) * a.n;
    const float* w_l[2] = {a.sorted_w + seg_s, a.sorted_w + seg_v};
    const float* m_l[2] = {a.sorted_m + seg_s, a.sorted_m + seg_v};
    const int32_t* i_l[2] = {a.sidx1 + seg_s, a.sidx1 + seg_v};
    if (tid == 0) { st.is = 0; st.iv = 0; st.ol_s = 0.f; st.ol_v = 0.f; st.sum = 0.f; st.done = 0; }
    __syncthreads();
    const float target = a.alpha * a.total[bh];
    const bool early = a.accounted == nullptr;
    while (true) {
        const int base_s = st.is, base_v = st.iv;          // windows start at the heads
        for (int l = 0; l < 2; ++l) {
            const int base = l == 0 ? base_s : base_v;
            for (int i = tid; i < WALK_CHUNK; i += WALK_THREADS) {
                const int gi = base + i;
                if (gi < n) {
                    const int64_t x = i_l[l][gi];
                    cw[l][i] = w_l[l][gi];
                    cm[l][i] = m_l[l][gi];
                    cl[l][i] = (float)((a.n - x) < nh ? (a.n - x) : nh);      // line length in the n_hat x n block
                }
            }
        }
        __syncthreads();
        if (tid == 0) {
            int is = base_s, iv = base_v;
            float ol_s = st.ol_s, ol_v = st.ol_v, sum = st.sum;
            // last index each head may reach inside this window (its successor must be loaded too)
            const int lim_s = (base_s + WALK_CHUNK >= n) ? n : base_s + WALK_CHUNK - 1;
            const int lim_v = (base_v + WALK_CHUNK >= n) ? n : base_v + WALK_CHUNK - 1;
            float ws = 0.f, ms = 0.f, ls = 0.f, wv = 0.f, mv = 0.f, lv = 0.f;          // heads
            float ws2 = 0.f, ms2 = 0.f, ls2 = 0.f, wv2 = 0.f, mv2 = 0.f, lv2 = 0.f;    // successors
            if (is < n) { ws = cw[0][0]; ms = cm[0][0]; ls = cl[0][0]; }
            if (is + 1 < n) { ws2 = cw[0][1]; ms2 = cm[0][1]; ls2 = cl[0][1]; }
            if (iv < n) { wv = cw[1][0]; mv = cm[1][0]; lv = cl[1][0]; }
            if (iv + 1 < n) { wv2 = cw[1][1]; mv2 = cm[1][1]; lv2 = cl[1][1]; }
            int done = 0;
            while (true) {
                if (!(sum < target) || (is >= n && iv >= n)) { done = 1; break; }
                if ((is < n && is >= lim_s) || (iv < n && iv >= lim_v)) break;          // slide the windows
                bool take_s;
                const float ds = __fsub_rn(ws, ol_v);
                const float dv = __fsub_rn(wv, ol_s);
                if (iv >= n) take_s = true;
                else if (is >= n) take_s = false;
                else {
                    float cs = __fsub_rn(ls, (float)iv); if (cs < 1.0f) cs = 1.0f;
                    float cv = __fsub_rn(lv, (float)is); if (cv < 1.0f) cv = 1.0f;
                    take_s = __fmul_rn(ds, cv) >= __fmul_rn(dv, cs);
                }
                if (early) {
                    // every later gain is <= the current head's (lists descend, overlaps only grow):
                    // if no available head has a positive gain the sum can never reach the target
                    const bool s_dead = (is >= n) || !(ds > 0.f);
                    const bool v_dead = (iv >= n) || !(dv > 0.f);
                    if (s_dead && v_dead) { is = n; iv = n; done = 1; break; }
                }
                if (take_s) {
                    sum = __fadd_rn(sum, ds); ol_s = __fadd_rn(ol_s, ms); ++is;
                    ws = ws2; ms = ms2; ls = ls2;
                    const int j = is + 1 - base_s;
                    if (is + 1 < n && j < WALK_CHUNK) { ws2 = cw[0][j]; ms2 = cm[0][j]; ls2 = cl[0][j]; }
                } else {
                    sum = __fadd_rn(sum, dv); ol_v = __fadd_rn(ol_v, mv); ++iv;
                    wv = wv2; mv = mv2; lv = lv2;
                    const int j = iv + 1 - base_v;
                    if (iv + 1 < n && j < WALK_CHUNK) { wv2 = cw[1][j]; mv2 = cm[1][j]; lv2 = cl[1][j]; }
                }
            }
            st.is = is; st.iv = iv; st.ol_s = ol_s; st.ol_v = ol_v; st.sum = sum; st.done = done;
        }
        __syncthreads();
        if (st.done) break;
    }
    if (tid == 0) {
        a.s_cnt[bh] = st.is;
        a.v_cnt[bh] = st.iv;
        if (a.accounted) a.accounted[bh] = st.sum;
    }
}

// ---- chosen prefix -> ascending index list --------------------------------------------------------
// grid (2, BH); dynamic LDS: bitmap of n bits + per-wave word counts.
__global__ __launch_bounds__(1024) void emit_kernel(SelectArgs a) {
    extern __shared__ uint32_t bm[];
    __shared__ uint32_t wsum[16];
    __shared__ uint32_t carry;
    const int list = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int64_t n = a.n;
    const int words = (int)((n + 31) / 32);
    const int64_t seg = ((int64_t)list * a.BH + bh) * n;
    const int32_t* sorted_idx = a.sidx1 + seg;
    const int cnt = list == 0 ? a.s_cnt[bh] : a.v_cnt[bh];
    int32_t* out = list == 0 ? a.s_idx + (int64_t)bh * a.cap_s : a.v_idx + (int64_t)bh * a.cap_v;
    const int cap = list == 0 ? a.cap_s : a.cap_v;
    for (int i = tid; i < words; i += 1024) bm[i] = 0u;
    if (tid == 0) carry = 0u;
    __syncthreads();
    for (int i = tid; i < cnt; i += 1024) { const int32_t x = sorted_idx[i]; atomicOr(&bm[x >> 5], 1u << (x & 31)); }
    __syncthreads();
    for (int w0 = 0; w0 < words; w0 += 1024) {
        const int wd = w0 + tid;
        const uint32_t m = wd < words ? bm[wd] : 0u;
        const uint32_t c = __popc(m);
        uint32_t inc = c;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) { const uint32_t t = __shfl_up(inc, off, 64); if (lane >= off) inc += t; }
        if (lane == 63) wsum[wv] = inc;
        __syncthreads();
        uint32_t pre = carry;
        for (int w = 0; w < wv; ++w) pre += wsum[w];
        uint32_t pos = pre + inc - c;
        uint32_t mm = m;
        while (mm) {
            const int bit = __ffs(mm) - 1;
            mm &= mm - 1;
            if (pos < (uint32_t)cap) out[pos] = wd * 32 + bit;
            ++pos;
        }
        __syncthreads();
        if (tid == 1023) carry = pre + inc;
        __syncthreads();
    }
}

// ---- top-B retention ------------------------------------------------------------------------------
// grid (B*Hkv).  keep_idx [BK][budget] ascending; keep_cnt = min(budget, len).
__global__ __launch_bounds__(1024) void topb_kernel(TopbArgs a) {
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sel_prefix, sel_remaining;
    __shared__ uint32_t wsum[16];
    __shared__ uint32_t carry_gt, carry_eq;
    const int bk = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int64_t len = a.len;
    const float* sc = a.score + (int64_t)bk * len;
    int32_t* out = a.keep_idx + (int64_t)bk * a.budget;
    const int64_t keep = a.budget < len ? a.budget : len;
    if (tid == 0) a.keep_cnt[bk] = (int32_t)keep;
    if (keep == len) {
        for (int64_t i = tid; i < len; i += 1024) out[i] = (int32_t)i;
        return;
    }
    // radix select on descending keys: find the key value K* of the keep-th element
    if (tid == 0) { sel_prefix = 0u; sel_remaining = (uint32_t)keep; }
    __syncthreads();
    for (int pass = 3; pass >= 0; --pass) {
        const int shift = 8 * pass;
        if (tid < 256) hist[tid] = 0u;
        __syncthreads();
        const uint32_t prefix = sel_prefix;
        const uint32_t himask = pass == 3 ? 0u : (0xFFFFFFFFu << (shift + 8));
        for (int64_t i = tid; i < len; i += 1024) {
            const uint32_t key = desc_key(sc[i]);
            if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t rem = sel_remaining, d = 0;
            for (; d < 256; ++d) { if (hist[d] >= rem) break; rem -= hist[d]; }
            sel_prefix = prefix | (d << shift);
            sel_remaining = rem;                       // how many elements equal to the prefix so far are still needed
        }
        __syncthreads();
    }
    const uint32_t kstar = sel_prefix;                 // smaller key = larger score
    const uint32_t need_eq = sel_remaining;            // elements with key == kstar to keep (smallest indices)
    if (tid == 0) { carry_gt = 0u; carry_eq = 0u; }
    __syncthreads();
    // ordered pass: position = (#kept before me); kept = key < kstar, or key == kstar among the first need_eq
    for (int64_t c0 = 0; c0 < len; c0 += 1024) {
        const int64_t i = c0 + tid;
        const uint32_t key = i < len ? desc_key(sc[i]) : 0xFFFFFFFFu;
        const uint32_t gt = (i < len && key < kstar) ? 1u : 0u;
        const uint32_t eq = (i < len && key == kstar) ? 1u : 0u;
        uint32_t v = gt | (eq << 16);                  // both counts in one scan (chunk <= 1024 < 65536)
        uint32_t inc = v;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) { const uint32_t t = __shfl_up(inc, off, 64); if (lane >= off) inc += t; }
        if (lane == 63) wsum[wv] = inc;
        __syncthreads();
        uint32_t pre = 0;
        for (int w = 0; w < wv; ++w) pre += wsum[w];
        const uint32_t ex = pre + inc - v;
        const uint32_t gt_before = carry_gt + (ex & 0xFFFFu), eq_before = carry_eq + (ex >> 16);
        const uint32_t eq_kept_before = eq_before < need_eq ? eq_before : need_eq;
        const bool kept = gt || (eq && eq_before < need_eq);
        if (kept) out[gt_before + eq_kept_before] = (int32_t)i;
        __syncthreads();
        if (tid == 1023) { const uint32_t tot = pre + inc; carry_gt += tot & 0xFFFFu; carry_eq += tot >> 16; }
        __syncthreads();
    }
}

// gather kept rows: dst [BK][budget][row_bytes] <- src [BK][len][row_bytes]; grid (budget, BK)
__global__ void gather_rows_kernel(const unsigned char* src, unsigned char* dst, const int32_t* keep_idx,
                                   const int32_t* keep_cnt, int64_t len, int budget, int row_bytes) {
    const int slot = blockIdx.x, bk = blockIdx.y;
    if (slot >= keep_cnt[bk]) return;
    const int64_t r = keep_idx[(int64_t)bk * budget + slot];
    const unsigned char* s = src + ((int64_t)bk * len + r) * row_bytes;
    unsigned char* d = dst + ((int64_t)bk * budget + slot) * row_bytes;
    for (int i = threadIdx.x * 16; i < row_bytes; i += blockDim.x * 16)
        *reinterpret_cast<f32x4*>(d + i) = *reinterpret_cast<const f32x4*>(s + i);
}

hipError_t run_select(const SelectArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(sort_kernel, dim3(2, a.BH), dim3(SORT_THREADS), 0, st, a);
    hipLaunchKernelGGL(walk_kernel, dim3(a.BH), dim3(WALK_THREADS), 0, st, a);
    const size_t smem = (size_t)((a.n + 31) / 32) * 4;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&emit_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(emit_kernel, dim3(2, a.BH), dim3(1024), smem, st, a);
    return hipGetLastError();
}

hipError_t run_topb(const TopbArgs& a, int BK, hipStream_t st) {
    hipLaunchKernelGGL(topb_kernel, dim3(BK), dim3(1024), 0, st, a);
    return hipGetLastError();
}

hipError_t run_gather_rows(const void* src, void* dst, const int32_t* keep_idx, const int32_t* keep_cnt,
                           int BK, int64_t len, int budget, int row_bytes, hipStream_t st) {
    hipLaunchKernelGGL(gather_rows_kernel, dim3(budget, BK), dim3(64), 0, st,
                       reinterpret_cast<const unsigned char*>(src), reinterpret_cast<unsigned char*>(dst),
                       keep_idx, keep_cnt, len, budget, row_bytes);
    return hipGetLastError();
}

}  // namespace ls
