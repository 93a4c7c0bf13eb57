// Sparse prefill attention over selected key columns and diagonals (gfx950).
//
// Computes, for every row a of the newest turn (absolute position p = n - n_hat + a),
//     out[a] = sum_b softmax_b( scale * <q_a, k_b> ) v_b   over the allowed cells
//     allowed(a, b)  <=>  b <= p  and  ( b is a selected column  or  p - b is a selected diagonal )
// which is the masked attention Softmax(QK^T/sqrt(d_k) - c(1 - M)) V of Sec. 2.2 with the mask M
// built from the vertical and slash lines chosen by Alg. 2 (Sec. 5.1), masked entries weighing zero.
//
// Work decomposition.  One workgroup (4 waves) owns 128 query rows of one (batch, head); blocks of
// rows are aligned to absolute positions that are multiples of 128, so the diagonals a 128 x 64 tile
// touches depend only on j = (row block start)/64 - (key block): offsets 64j - 63 .. 64j + 127.  A
// per-head table built by plan_kernel says, for each j, whether any (or every) diagonal in that range
// is selected.
//   phase 1: key blocks whose diagonal range holds a selected diagonal are streamed as contiguous
//            64-key tiles; the cell mask is the diagonal bit, read from a bitmap in LDS.
//   phase 2: the selected columns (up to the block's last row) are gathered, 64 at a time, into
//            packed tiles; a cell is dropped there if its diagonal is selected (phase 1 counted it),
//            which the per-j table decides for whole columns in the common cases.
// So every allowed cell is visited exactly once.  Each wave owns 32 rows and skips the 32 x 32
// sub-tiles in which none of its rows has an allowed cell.
//
// Tile products: S^T = K_tile * Q^T and O^T += V_tile^T * P^T on 32x32 MFMA, fp32 accumulation,
// online softmax in the base-2 domain.  K is staged row-major in LDS, V transposed (see vt_col).
#include <type_traits>
#include <hip/hip_ext.h>
#include "ls_device.h"
#include "ls_internal.h"

namespace ls {

#ifndef LS_RING_S
#define LS_RING_S 4       // K fragments in flight ahead of the QK^T products
#endif
#ifndef LS_RING_P
#define LS_RING_P 3       // V^T fragments in flight ahead of the P*V products
#endif
constexpr int BM = 128;   // query rows per workgroup
constexpr int BN = 64;    // keys per tile
constexpr int PREFILL_THREADS = 256;

// ---------------------------------------------------------------------------------------------
// plan: per (batch, head) bitmap of the selected diagonals, the per-j activity table, a head flag.
//   obits : [BH][words + 1] uint32: one zero word, then bit o in word 1 + o/32; words = n/32 rounded up + 8 zero words
//   tab   : [BH][tab_len] bytes, entry j+1 for j = -1 .. ; bit0 = some diagonal of
//           [64j-63, 64j+127] is selected, bit1 = all of them are (and none is cut off at 0 or n-1)
//   hflag : [BH] bytes, bit0 = every diagonal 0..n-1 is selected (the mask is plain causal),
//           bit1 = the column list is not strictly ascending inside [0, n): its columns are ignored
// ---------------------------------------------------------------------------------------------
// Exclusive prefix sum over the 1024 threads of a workgroup (wave shuffles + one LDS round).
// `wsum` must hold 16 words; returns the sum of `v` over the threads before this one and, in
// `total`, the sum over all threads.
__device__ __forceinline__ uint32_t block_scan_1024(uint32_t v, uint32_t* wsum, uint32_t& total) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) { const uint32_t t = __shfl_up(inc, off, 64); if (lane >= off) inc += t; }
    __syncthreads();                                       // wsum may still be read from an earlier call
    if (lane == 63) wsum[wv] = inc;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) { const uint32_t t = wsum[w]; all += t; if (w < wv) before += t; }
    total = all;
    return before + inc - v;
}

constexpr int LS_MAX_TAB = 262144 / 64 + 8;  // table entries at the largest supported context
__global__ __launch_bounds__(1024) void plan_kernel(PlanArgs a) {
    extern __shared__ uint32_t sm[];
    __shared__ int total_bits;
    __shared__ uint8_t tabs[LS_MAX_TAB];
    const int bh = blockIdx.x;
    const int64_t n = a.n;
    const int words = a.words;
    const int tid = threadIdx.x;
    int ns = a.s_cnt[bh]; if (ns > a.cap_s) ns = a.cap_s; if (ns < 0) ns = 0;
    const int32_t* si = a.s_idx + (int64_t)bh * a.cap_s;
    for (int i = tid; i < words; i += blockDim.x) sm[i] = 0u;
    if (tid == 0) total_bits = 0;
    // The column list must be strictly ascending and inside [0, n) (the attention kernel bisects it and
    // gathers K / V rows through it): a head whose list is not has its columns ignored (hflag bit 1) and the
    // context's status word says so.  Diagonals outside [0, n) are skipped below and reported likewise.
    int nvl = a.v_cnt[bh]; if (nvl > a.cap_v) nvl = a.cap_v; if (nvl < 0) nvl = 0;
    const int32_t* vl = a.v_idx + (int64_t)bh * a.cap_v;
    bool v_bad = false, s_bad = false;
    if ((reinterpret_cast<uintptr_t>(vl) & 15) == 0 && a.cap_v % 4 == 0) {     // four entries per load (and the one before them)
        typedef __attribute__((ext_vector_type(4))) int32_t i32x4;
        for (int i0 = 4 * tid; i0 < nvl; i0 += 4 * (int)blockDim.x) {
            const i32x4 c4 = *reinterpret_cast<const i32x4*>(vl + i0);     // entries past nvl (inside the capacity, a multiple of 4 here) are not looked at
            int32_t prev = i0 > 0 ? vl[i0 - 1] : -1;
            const int32_t c[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (i0 + e < nvl) { v_bad = v_bad || c[e] <= prev || c[e] >= n; prev = c[e]; }
            }
        }
    } else {
        for (int i = tid; i < nvl; i += blockDim.x) {
            const int32_t c = vl[i];
            v_bad = v_bad || c < 0 || c >= n || (i > 0 && vl[i - 1] >= c);
        }
    }
    v_bad = __syncthreads_or(v_bad);
    // every diagonal selected (a head the walk gave up sparsifying): the list is 0 .. n-1, checked while it is read
    bool ident = ns == (int)n;
    if (ident) {
        for (int i0 = tid; i0 < ns; i0 += 8 * 1024) {
            int32_t o8[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) { const int i = i0 + j * 1024; o8[j] = i < ns ? si[i] : i; }
#pragma unroll
            for (int j = 0; j < 8; ++j) ident = ident && o8[j] == i0 + j * 1024;
        }
        ident = __syncthreads_and(ident);
        if (ident) for (int i = tid; i < (int)((n + 31) / 32); i += blockDim.x) sm[i] = (i == (int)(n / 32)) ? ((1u << (n & 31)) - 1u) : 0xFFFFFFFFu;
    }
    for (int i0 = tid; i0 < (ident ? 0 : ns); i0 += 8 * 1024) {          // eight independent loads in flight per thread
        int32_t o8[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) { const int i = i0 + j * 1024; o8[j] = i < ns ? si[i] : -1; }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            // The list is ascending, so neighbouring lanes mostly hit the same bitmap word: their bits are OR-ed
            // across each run of equal words inside a row of 16 lanes first (four doubling steps of row shifts,
            // plain vector moves) and the run's first lane, and every 16th lane, does the one atomic.  Correct for
            // any order of the list.
            const bool ok = o8[j] >= 0 && o8[j] < n;
            s_bad = s_bad || (!ok && i0 + j * 1024 < ns);
            const int wd = ok ? o8[j] >> 5 : -1 - (tid & 63);
            uint32_t m = ok ? 1u << (o8[j] & 31) : 0u;
            // value of the lane `off` to the right inside the row (lanes shifted in from outside a row read -2 / 0)
#define LS_ROW_SHL(x, off, fill) __builtin_amdgcn_update_dpp((int)(fill), (int)(x), 0x100 + (off), 0xF, 0xF, false)
#define LS_OR_STEP(off) { const uint32_t tm = (uint32_t)LS_ROW_SHL(m, off, 0); const int tw = LS_ROW_SHL(wd, off, -2); if (tw == wd) m |= tm; }
            LS_OR_STEP(1) LS_OR_STEP(2) LS_OR_STEP(4) LS_OR_STEP(8)
            const int pw = __builtin_amdgcn_update_dpp(-2, wd, 0x110 + 1 /* row_shr:1 */, 0xF, 0xF, false);
#undef LS_OR_STEP
#undef LS_ROW_SHL
            if (ok && pw != wd) atomicOr(&sm[wd], m);
        }
    }
    __syncthreads();
    int mine = 0;
    uint32_t* og = a.obits + (int64_t)bh * (words + 1);       // one zero word, then the bitmap
    if (tid == 0) og[0] = 0u;
    for (int i = tid; i < words; i += blockDim.x) { og[i + 1] = sm[i]; mine += __popc(sm[i]); }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mine += __shfl_down(mine, off, 64);       // one atomic per wave, not per thread
    if ((tid & 63) == 0) atomicAdd(&total_bits, mine);
    // activity table
    for (int e = tid; e < a.tab_len; e += blockDim.x) {
        const int64_t j = (int64_t)e - 1;
        int64_t lo = 64 * j - 63, hi = 64 * j + 127;
        const bool cut = lo < 0;
        if (lo < 0) lo = 0;
        if (hi > n - 1) hi = n - 1;
        int cnt = 0;
        if (hi >= lo) {
            const int w0 = (int)(lo >> 5), w1 = (int)(hi >> 5);
            for (int wd = w0; wd <= w1; ++wd) {
                uint32_t m = sm[wd];
                if (wd == w0) m &= 0xFFFFFFFFu << (lo & 31);
                if (wd == w1) m &= 0xFFFFFFFFu >> (31 - (hi & 31));
                cnt += __popc(m);
            }
        }
        uint8_t f = 0;
        if (cnt > 0) f |= 1;
        if (!cut && hi >= lo && cnt == (int)(hi - lo + 1) && hi == 64 * j + 127) f |= 2;
        a.tab[(int64_t)bh * a.tab_len + e] = f;
        tabs[e] = f;                                       // LDS copy for the counts below
    }
    __syncthreads();
    // prefix counts of active entries: pref[e] = number of active entries below e
    __shared__ uint32_t wsum[16];
    const int chunk = (a.tab_len + (int)blockDim.x - 1) / (int)blockDim.x;
    const int e0 = tid * chunk < a.tab_len ? tid * chunk : a.tab_len, e1 = (e0 + chunk < a.tab_len) ? e0 + chunk : a.tab_len;
    int mine2 = 0;
    for (int e = e0; e < e1; ++e) mine2 += tabs[e] & 1;
    uint32_t active_entries;
    uint32_t run = block_scan_1024((uint32_t)mine2, wsum, active_entries);
    uint16_t* pref = a.pref + (int64_t)bh * (a.tab_len + 1);
    for (int e = e0; e < e1; ++e) { pref[e] = (uint16_t)run; run += tabs[e] & 1; }
    if (e1 == a.tab_len && e0 < a.tab_len) pref[a.tab_len] = (uint16_t)run;
    // head flag and cost estimate: table entries with a selected diagonal (key blocks a late row block
    // visits) plus packed column tiles
    s_bad = __syncthreads_or(s_bad);
    if (tid == 0) {
        a.hflag[bh] = ((total_bits == (int)n) ? 1 : 0) | (v_bad ? 2 : 0);
        if (v_bad) atomicOr(a.status, STAT_V_INVALID);
        if (s_bad) atomicOr(a.status, STAT_S_RANGE);
        int nv = a.v_cnt[bh]; if (nv > a.cap_v) nv = a.cap_v; if (nv < 0) nv = 0;
        if (total_bits == (int)n || v_bad) nv = 0;
        a.cost[bh] = (uint32_t)((int)active_entries + (nv + 63) / 64 + 1);
    }
}

// ---------------------------------------------------------------------------------------------
// sched: builds the 8 work queues.  The query heads of one KV head stay together (they share K/V
// tiles in one L2); KV groups are dealt to the XCDs heaviest first, each to the XCD with the least
// work so far.
// One workgroup per queue; groups beyond SCHED_MAX_GROUPS fall back to round-robin dealing.  Inside a
// queue items are ordered by decreasing tile count, so the long ones start first.
// ---------------------------------------------------------------------------------------------
constexpr int SCHED_MAX_GROUPS = 2048;
constexpr int SCHED_MAX_HEADS = 8192;      // heads one XCD's queue can take
constexpr int SCHED_THREADS = 1024;
__global__ __launch_bounds__(SCHED_THREADS) void sched_kernel(SchedArgs a) {
    __shared__ uint32_t gcost[SCHED_MAX_GROUPS];
    __shared__ uint16_t order[SCHED_MAX_GROUPS];          // groups by decreasing cost
    __shared__ uint16_t bin_of[SCHED_MAX_GROUPS];
    const int tid = threadIdx.x;
    const int groups = a.BH / a.G;
    const bool sorted = groups <= SCHED_MAX_GROUPS;
    if (sorted) {                                          // every block repeats this small computation
        for (int gi = tid; gi < groups; gi += SCHED_THREADS) {
            const int b = gi / a.Hkv, kvh = gi % a.Hkv;
            uint32_t c = 0;
            for (int g = 0; g < a.G; ++g) c += a.cost[b * a.Hq + kvh * a.G + g];
            gcost[gi] = c;
        }
        __syncthreads();
        for (int gi = tid; gi < groups; gi += SCHED_THREADS) {   // rank sort (ties: smaller index first)
            const uint32_t c = gcost[gi];
            int rank = 0;
            for (int o = 0; o < groups; ++o) { const uint32_t d = gcost[o]; rank += (d > c) || (d == c && o < gi); }
            order[rank] = (uint16_t)gi;
        }
        __syncthreads();
        if (tid == 0) {
            uint64_t load[8];
            for (int x = 0; x < 8; ++x) load[x] = 0;
            for (int r = 0; r < groups; ++r) {
                const int gi = order[r];
                int best = 0;
                for (int x = 1; x < 8; ++x) if (load[x] < load[best]) best = x;
                bin_of[gi] = (uint16_t)best;
                load[best] += gcost[gi] + 1;
            }
        }
        __syncthreads();
    }
    // Work items (head, row block) of this block's bin, heaviest first.  Item cost = key blocks with a
    // selected diagonal that the row block visits (from the prefix counts) + packed column tiles.
    __shared__ uint32_t hist[4097];
    __shared__ uint16_t heads[SCHED_MAX_HEADS];
    __shared__ int nheads;
    const int x = blockIdx.x;
    const int64_t qcap = (int64_t)a.BH * a.nqb;
    auto item_cost = [&](int bh, int qb) -> int {
        const int64_t blockpos = a.pos0 + (int64_t)qb * BM;
        const int64_t posmax = (blockpos + BM - 1 < a.n - 1) ? blockpos + BM - 1 : a.n - 1;
        const int jb = (int)(blockpos / BN), kb_hi = (int)(posmax / BN);
        const uint16_t* pref = a.pref + (int64_t)bh * (a.tab_len + 1);
        int c = pref[jb + 2] - pref[jb - kb_hi + 1];      // entries jb-kb_hi+1 .. jb+1
        int nv = a.v_cnt[bh]; if (nv > a.cap_v) nv = a.cap_v; if (nv < 0) nv = 0;
        if (a.hflag[bh] & 3) nv = 0;
        c += (nv + 63) / 64;
        return c > 4095 ? 4095 : c;
    };
    for (int i = tid; i < 4097; i += SCHED_THREADS) hist[i] = 0u;
    if (tid == 0) nheads = 0;
    __syncthreads();
    for (int bh = tid; bh < a.BH; bh += SCHED_THREADS) {   // heads of this bin (order inside the list is free)
        const int b = bh / a.Hq, h = bh % a.Hq, gi = b * a.Hkv + h / a.G;
        const int bin = sorted ? (int)bin_of[gi] : (gi & 7);
        if (bin == x) { const int i = atomicAdd(&nheads, 1); if (i < SCHED_MAX_HEADS) heads[i] = (uint16_t)bh; }
    }
    __syncthreads();
    const int nh_ = nheads < SCHED_MAX_HEADS ? nheads : SCHED_MAX_HEADS;
    const int64_t items = (int64_t)nh_ * a.nqb;
    for (int64_t it = tid; it < items; it += SCHED_THREADS)
        atomicAdd(&hist[4095 - item_cost(heads[it / a.nqb], (int)(it % a.nqb))], 1u);
    __syncthreads();
    {                                                      // exclusive scan in decreasing-cost order
        __shared__ uint32_t wsum[16];
        uint32_t h4[4], mine = 0, all;
#pragma unroll
        for (int q = 0; q < 4; ++q) { h4[q] = hist[4 * tid + q]; mine += h4[q]; }
        uint32_t run = block_scan_1024(mine, wsum, all);
#pragma unroll
        for (int q = 0; q < 4; ++q) { hist[4 * tid + q] = run; run += h4[q]; }
    }
    __syncthreads();
    for (int64_t it = tid; it < items; it += SCHED_THREADS) {
        const int bh = heads[it / a.nqb], qb = (int)(it % a.nqb);
        const uint32_t posn = atomicAdd(&hist[4095 - item_cost(bh, qb)], 1u);
        a.queue[(int64_t)x * qcap + posn] = ((uint32_t)bh << 16) | (uint32_t)qb;
    }
    if (tid == 0) { a.qlen[x] = (int)items; a.qhead[x] = 0; }
}

// Persistent launch: enough workgroups to fill the chip at any occupancy this kernel reaches
// (256 CUs x up to 4 resident workgroups); surplus workgroups find the queues empty and leave.
static int persistent_grid(const PrefillArgs& a) {
    const int64_t total = (int64_t)a.BH * a.nqb;
    return (int)(total < 1024 ? total : 1024);
}

// Next work item for this workgroup: its own XCD's queue first, then the others in ring order.
// Returns -1 when every queue is drained (each queue hands out each item once; the scan is finite).
__device__ __forceinline__ int pop_item(const PrefillArgs& a, int my_x) {
    for (int k = 0; k < 8; ++k) {
        const int x = (my_x + k) & 7;
        const int len = a.qlen[x];
        if (__atomic_load_n(&a.qhead[x], __ATOMIC_RELAXED) < len) {
            const int i = atomicAdd(&a.qhead[x], 1);
            if (i < len) return (int)a.queue[(int64_t)x * a.qcap + i];
        }
    }
    return -1;
}

// ---------------------------------------------------------------------------------------------
// the attention kernel
// ---------------------------------------------------------------------------------------------
template <typename T, int D>
struct TileCfg {
    static constexpr int EB = Elem<T>::bytes;
    static constexpr int EPC = Elem<T>::per16;            // elements per 16-byte chunk
    static constexpr int CPR = D / EPC;                   // 16-byte chunks per K/V row
    static constexpr int CPT = CPR / 4;                   // chunks each thread moves per tile and operand
    static constexpr int K_STRIDE = D * EB + 16;          // bytes per staged K row
    static constexpr int VT_STRIDE = BN * EB + 16;        // bytes per staged V^T row
    static constexpr int K_BYTES = BN * K_STRIDE;
    static constexpr int VT_BYTES = D * VT_STRIDE;
    static constexpr int KSTEPS = D / 16;                 // k chunks of the QK^T product
    static constexpr int DBLK = D / 32;                   // 32-wide output column blocks
};

template <typename T>
__device__ __forceinline__ void store_vt(unsigned char* vt, int stride, int d0, int col, const f32x4 raw);

// raw holds 16 bytes of one V row: elements d0 .. d0+EPC-1; scatter them down column `col`.
template <>
__device__ __forceinline__ void store_vt<bf16_t>(unsigned char* vt, int stride, int d0, int col, const f32x4 raw) {
    struct U4 { uint32_t w[4]; } u = __builtin_bit_cast(U4, raw);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        *reinterpret_cast<uint16_t*>(vt + (d0 + 2 * i) * stride + col * 2) = (uint16_t)(u.w[i] & 0xFFFFu);
        *reinterpret_cast<uint16_t*>(vt + (d0 + 2 * i + 1) * stride + col * 2) = (uint16_t)(u.w[i] >> 16);
    }
}
template <>
__device__ __forceinline__ void store_vt<float>(unsigned char* vt, int stride, int d0, int col, const f32x4 raw) {
    *reinterpret_cast<float*>(vt + (d0 + 0) * stride + col * 4) = raw.x;
    *reinterpret_cast<float*>(vt + (d0 + 1) * stride + col * 4) = raw.y;
    *reinterpret_cast<float*>(vt + (d0 + 2) * stride + col * 4) = raw.z;
    *reinterpret_cast<float*>(vt + (d0 + 3) * stride + col * 4) = raw.w;
}

__device__ __forceinline__ void store_out4(bf16_t* p, float a, float b, float c, float d) {
    struct U2 { uint32_t x, y; } u;
    u.x = (uint32_t)f2bf(a) | ((uint32_t)f2bf(b) << 16);
    u.y = (uint32_t)f2bf(c) | ((uint32_t)f2bf(d) << 16);
    *reinterpret_cast<U2*>(p) = u;
}
__device__ __forceinline__ void store_out4(float* p, float a, float b, float c, float d) {
    const f32x4 v = {a, b, c, d};
    *reinterpret_cast<f32x4*>(p) = v;
}

// 32 consecutive bits of a bitmap starting at bit `base` (may be negative: those bits read 0).
// `bits1` is the bitmap preceded by one zero word (bits1[i + 1] = word i), which makes this branch-free.
__device__ __forceinline__ uint32_t window32(const uint32_t* bits1, int64_t base) {
    const int b32 = (int)(base < -32 ? -32 : base) + 32;     // >= 0, bit index in the padded map
    const int wd = b32 >> 5, sh = b32 & 31;
    const uint64_t x = (uint64_t)bits1[wd] | ((uint64_t)bits1[wd + 1] << 32);
    return (uint32_t)(x >> sh);
}

// Tile sequence of one workgroup: first the n1 key blocks crossed by a selected diagonal (ascending),
// then n2 packed tiles of 64 selected columns each.  K/V rows of tile t+1 are fetched into registers
// while tile t is multiplied out of LDS buffer t&1, then written to buffer (t+1)&1; one barrier per tile.
template <typename T, int D>
__global__ __launch_bounds__(PREFILL_THREADS, 2) void prefill_kernel(PrefillArgs a) {
    using C = TileCfg<T, D>;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* k_lds = smem;                                         // [2][K_BYTES]
    unsigned char* vt_lds = smem + 2 * C::K_BYTES;                       // [2][VT_BYTES]
    uint32_t* ob = reinterpret_cast<uint32_t*>(smem + 2 * C::K_BYTES + 2 * C::VT_BYTES);
    int32_t* colring = reinterpret_cast<int32_t*>(ob + a.words + 1);     // [2][64]; ob = zero word + bitmap
    int32_t* wcnt = colring + 128;                                       // [8]
    uint16_t* kbl = reinterpret_cast<uint16_t*>(wcnt + 8);               // [tab_len] active key blocks
    uint8_t* tab = reinterpret_cast<uint8_t*>(kbl + ((a.tab_len + 7) & ~7));

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r32 = lane & 31, g = lane >> 5;

    __shared__ int item_s;
  for (;;) {                                               // persistent: one (head, row block) item per trip
    __syncthreads();                                       // everyone is done with the previous item's LDS
    if (tid == 0) item_s = pop_item(a, blockIdx.x & 7);    // taken only when needed: items are coarse, reserving early hurts the tail
    __syncthreads();
    const int item = item_s;
    if (item < 0) break;
    const int bh = item >> 16, qb = item & 0xFFFF;
    const int b = bh / a.Hq, h = bh % a.Hq, kvh = h / a.G;
    const int64_t n = a.n, row0 = n - a.n_hat;
    const int64_t blockpos = a.pos0 + (int64_t)qb * BM;                  // multiple of 128
    const int64_t posmax = (blockpos + BM - 1 < n - 1) ? blockpos + BM - 1 : n - 1;
    const T* Kg = reinterpret_cast<const T*>(a.k) + ((int64_t)b * a.Hkv + kvh) * n * D;
    const T* Vg = reinterpret_cast<const T*>(a.v) + ((int64_t)b * a.Hkv + kvh) * n * D;
    const T* Qg = reinterpret_cast<const T*>(a.q) + (int64_t)bh * a.n_hat * D;

    // diagonal bitmap and activity table of this head -> LDS
    for (int i = tid; i < a.words + 1; i += PREFILL_THREADS) ob[i] = a.obits[(int64_t)bh * (a.words + 1) + i];
    for (int i = tid; i < a.tab_len; i += PREFILL_THREADS) tab[i] = a.tab[(int64_t)bh * a.tab_len + i];

    // this lane's query row and its fragments
    const int64_t pos = blockpos + 32 * wv + r32;
    const bool row_ok = (pos >= row0) && (pos < n);
    Frag<T> qf[C::KSTEPS];
    if (row_ok) {
        const T* qrow = Qg + (pos - row0) * D;
#pragma unroll
        for (int c = 0; c < C::KSTEPS; ++c) load_frag(qf[c], qrow + 16 * c + 8 * g);
    } else {
#pragma unroll
        for (int c = 0; c < C::KSTEPS; ++c) zero_frag(qf[c]);
    }
    __syncthreads();

    // ---- ordered list of the key blocks phase 1 visits
    const int64_t jb = blockpos / BN;                      // even
    const int kb_hi = (int)(posmax / BN);
    int n1 = 0;
    for (int base = 0; base <= kb_hi; base += PREFILL_THREADS) {
        const int kb = base + tid;
        const bool act = kb <= kb_hi && (tab[jb - kb + 1] & 1);
        const uint64_t bal = __ballot(act);
        if (lane == 0) wcnt[wv] = __popcll(bal);
        __syncthreads();
        int off = n1;
        for (int w2 = 0; w2 < wv; ++w2) off += wcnt[w2];
        if (act) kbl[off + __popcll(bal & ((1ull << lane) - 1ull))] = (uint16_t)kb;
        n1 += wcnt[0] + wcnt[1] + wcnt[2] + wcnt[3];
        __syncthreads();
    }
    // ---- how many selected columns phase 2 gathers (columns beyond the block's last row are invisible)
    int nv = a.v_cnt[bh]; if (nv > a.cap_v) nv = a.cap_v; if (nv < 0) nv = 0;
    const int32_t* vi = a.v_idx + (int64_t)bh * a.cap_v;
    if (a.hflag[bh] & 3) nv = 0;                           // every diagonal is selected (phase 1 covers all cells), or the list is unusable
    if (nv > 0 && (int64_t)vi[nv - 1] > posmax) {          // ascending list: binary search for the first column > posmax
        int lo = 0, hi = nv - 1;
        while (lo < hi) { const int mid = (lo + hi) >> 1; if ((int64_t)vi[mid] > posmax) hi = mid; else lo = mid + 1; }
        nv = lo;
    }
    const int n2 = (nv + BN - 1) / BN;
    const int ntiles = n1 + n2;

    f32x16 oacc[C::DBLK];
#pragma unroll
    for (int i = 0; i < C::DBLK; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;                  // m_run in raw logit units
    const float sc2 = a.scale_log2e;

    // ---- one staged tile: masks am0 / am1 say which of the 2 x 32 keys this lane's row may see
    auto process = [&](const unsigned char* kt, const unsigned char* vt, uint32_t am0, uint32_t am1, bool full) {
        f32x16 s[2];
        bool act[2];
        act[0] = __ballot(am0 != 0u) != 0ull;
        act[1] = __ballot(am1 != 0u) != 0ull;
        if (!act[0] && !act[1]) return;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[sub][r] = 0.f;
            if (act[sub]) {
                const unsigned char* krow = kt + (32 * sub + r32) * C::K_STRIDE + 8 * g * C::EB;
#pragma unroll
                for (int c = 0; c < C::KSTEPS; ++c) {
                    Frag<T> kf;
                    load_frag(kf, krow + 16 * c * C::EB);
                    mma(s[sub], kf, qf[c]);        // s[r] = <k_{8(r/4)+4g+r%4}, q_row>
                }
            }
        }
        float mx = -INFINITY;
        if (full) {
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[sub][r]);
        } else {
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const uint32_t am = sub ? am1 : am0;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int kbit = 8 * (r >> 2) + 4 * g + (r & 3);
                    const float x = ((am >> kbit) & 1u) ? s[sub][r] : -INFINITY;
                    s[sub][r] = x;
                    mx = fmaxf(mx, x);
                }
            }
        }
        mx = fmaxf(mx, xor32(mx));
        const float m_new = fmaxf(m_run, mx);
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        const float corr = fast_exp2((m_run - m_safe) * sc2);
        const float mneg = -m_safe * sc2;
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = fast_exp2(__builtin_fmaf(s[sub][r], sc2, mneg));
                s[sub][r] = p;
                psum += p;
            }
        l_run = l_run * corr + psum;
        if (__ballot(corr != 1.0f) != 0ull) {
#pragma unroll
            for (int i = 0; i < C::DBLK; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[i][r] *= corr;
        }
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            if (!act[sub]) continue;
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                float pv[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) pv[e] = s[sub][8 * hh + e];
                Frag<T> pf;
                pack_frag(pf, pv);
#pragma unroll
                for (int i = 0; i < C::DBLK; ++i) {
                    Frag<T> vf;
                    load_frag(vf, vt + (32 * i + r32) * C::VT_STRIDE + (32 * sub + 16 * hh + 8 * g) * C::EB);
                    mma(oacc[i], vf, pf);          // O^T[d][row] += V^T[d][key] P^T[key][row]
                }
            }
        }
    };

    // ---- staging: thread -> (row tid/4, chunks tid%4 + 4i) for K, (row tid%64, chunks (tid/64)*CPT + i) for V
    const int rk = tid >> 2, ck0 = tid & 3;
    const int rv = tid & 63, cv0 = (tid >> 6) * C::CPT;
    const int vcol = vt_col(rv);
    f32x4 kreg[C::CPT], vreg[C::CPT];
    int32_t colk = -1, colv = -1;                          // gathered rows of the tile being fetched

    // global row feeding slot r of tile t (or -1): contiguous tiles read key block kbl[t]
    auto src_row = [&](int t, int r, int32_t gathered) -> int64_t {
        if (t < n1) { const int64_t kr = (int64_t)kbl[t] * BN + r; return kr < n ? kr : -1; }
        return gathered;
    };
    auto load_cols = [&](int t) {                          // column indices of gathered tile t -> registers
        colk = -1; colv = -1;
        if (t >= n1 && t < ntiles) {
            const int base = (t - n1) * BN;
            if (base + rk < nv) colk = vi[base + rk];
            if (base + rv < nv) colv = vi[base + rv];
        }
    };
    auto fetch = [&](int t) {                              // global -> registers, no divergent branches
        const int64_t gk = src_row(t, rk, colk), gv = src_row(t, rv, colv);
        const unsigned char* pk = reinterpret_cast<const unsigned char*>(Kg + (gk < 0 ? 0 : gk) * D) + 16 * ck0;
        const unsigned char* pv = reinterpret_cast<const unsigned char*>(Vg + (gv < 0 ? 0 : gv) * D) + 16 * cv0;
#pragma unroll
        for (int i = 0; i < C::CPT; ++i) {
            kreg[i] = *reinterpret_cast<const f32x4*>(pk + 64 * i);
            vreg[i] = *reinterpret_cast<const f32x4*>(pv + 16 * i);
        }
        if (__ballot(gk < 0 || gv < 0) != 0ull) {          // a slot without a row (tail of the context or of the list)
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < C::CPT; ++i) {
                if (gk < 0) kreg[i] = z;
                if (gv < 0) vreg[i] = z;
            }
        }
    };
    auto stash = [&](int t) {                              // registers -> LDS buffer t & 1 (+ column ids)
        unsigned char* kt = k_lds + (t & 1) * C::K_BYTES;
        unsigned char* vt = vt_lds + (t & 1) * C::VT_BYTES;
#pragma unroll
        for (int i = 0; i < C::CPT; ++i) {
            *reinterpret_cast<f32x4*>(kt + rk * C::K_STRIDE + 16 * (ck0 + 4 * i)) = kreg[i];
            store_vt<T>(vt, C::VT_STRIDE, (cv0 + i) * C::EPC, vcol, vreg[i]);
        }
        if (t >= n1 && tid < BN) colring[(t & 1) * BN + tid] = colv;
    };

    if (ntiles > 0) {
        load_cols(0);
        fetch(0);
        stash(0);
        load_cols(1);
    }
    __syncthreads();

    for (int t = 0; t < ntiles; ++t) {
        const bool more = t + 1 < ntiles;
        if (more) fetch(t + 1);                            // uses the columns loaded one iteration ago
        const int32_t colv_next = colv;
        if (more) load_cols(t + 2);
        // ---- masks of tile t
        uint32_t am0 = 0u, am1 = 0u;
        bool full = false;
        if (t < n1) {
            const int64_t key0 = (int64_t)kbl[t] * BN;
            const uint8_t f = tab[jb - kbl[t] + 1];
            if (!row_ok) { am0 = am1 = 0u; }
            else if (f & 2) { am0 = am1 = 0xFFFFFFFFu; }
            else {
                // bit i of the mask <-> key key0 + 32*sub + i <-> diagonal pos - key
                const int64_t d0 = pos - key0;             // diagonal of the tile's first key
                am0 = __brev(window32(ob, d0 - 31));
                am1 = __brev(window32(ob, d0 - 63));
            }
            full = (f & 2) && (__ballot(row_ok) == ~0ull);
        } else {
            const int32_t* cols = colring + (t & 1) * BN;
            const int base = (t - n1) * BN;
            const int cnt = nv - base < BN ? nv - base : BN;
            // slot `lane`: is the column's key block crossed by selected diagonals for this row block?
            const int32_t mycol = lane < cnt ? cols[lane] : 0;
            const uint8_t f = lane < cnt ? tab[jb - (mycol >> 6) + 1] : (uint8_t)3;
            const uint64_t drop = __ballot(f == 3);        // wholly covered by phase 1 (or no such slot)
            const uint64_t chk = __ballot(f == 1);         // partly covered: test cell by cell
            uint64_t am = 0ull;
            if (row_ok) {
                // causal: columns ascend, the visible ones form a prefix
                if ((int64_t)cols[cnt - 1] <= pos) am = cnt >= 64 ? ~0ull : ((1ull << cnt) - 1ull);
                else for (int i = 0; i < cnt; ++i) if ((int64_t)cols[i] <= pos) am |= 1ull << i;
                am &= ~drop;
                uint64_t todo = chk & am;
                while (todo) {
                    const int i = __ffsll((unsigned long long)todo) - 1;
                    todo &= todo - 1;
                    const int64_t o = pos - cols[i];       // >= 0 here
                    if ((ob[(o >> 5) + 1] >> (o & 31)) & 1u) am &= ~(1ull << i);   // cell already counted on its diagonal
                }
            }
            am0 = (uint32_t)am; am1 = (uint32_t)(am >> 32);
        }
        process(k_lds + (t & 1) * C::K_BYTES, vt_lds + (t & 1) * C::VT_BYTES, am0, am1, full);
        if (more) {
            const int32_t keep = colv; colv = colv_next;   // stash() records the columns of tile t+1
            stash(t + 1);
            colv = keep;
        }
        __syncthreads();
    }

    // ================= epilogue =================
    const float l_tot = l_run + xor32(l_run);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    if (row_ok) {
        T* orow = reinterpret_cast<T*>(a.out) + ((int64_t)bh * a.n_hat + (pos - row0)) * D;
#pragma unroll
        for (int i = 0; i < C::DBLK; ++i)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int d0 = 32 * i + 8 * rq + 4 * g;
                store_out4(orow + d0, oacc[i][4 * rq] * inv, oacc[i][4 * rq + 1] * inv,
                           oacc[i][4 * rq + 2] * inv, oacc[i][4 * rq + 3] * inv);
            }
        if (a.lse && g == 0)
            a.lse[(int64_t)bh * a.n_hat + (pos - row0)] =
                l_tot > 0.f ? (m_run * sc2 + log2f(l_tot)) * 0.69314718055994531f : -INFINITY;
    }
  }                                                        // next item
}

// ---------------------------------------------------------------------------------------------
// bf16 kernel: same tile sequence, masks and softmax as prefill_kernel, but staged the CDNA4 way.
//   * K and V rows go straight from global memory into LDS (global_load_lds, 16 bytes per lane, no
//     registers, no LDS store instructions).  A lane's 16 bytes land at LDS base + 16 * lane, so one
//     wave-wide transfer fills 1024 consecutive bytes: RPI whole rows of DS 16-byte slots.  Where a
//     lane's bytes land is fixed; which bytes it fetches is free, so slot s of row r receives chunk
//     s ^ swizzle(r) of that row.  The swizzles (kswz, vswz) are chosen so that the fragment reads
//     below touch every LDS bank once per pass; for d = 128 the K transfers are also spaced 64 bytes
//     apart.  All transfers of a wave then differ only in a uniform base address: one per-lane
//     offset register per operand serves the whole kernel.
//   * V stays row-major; the V^T fragments of the P*V product come from the LDS transpose read
//     ds_read_b64_tr_b16: in a block of 16 lanes, lane s addresses 4 consecutive 16-bit values and
//     lane L receives value L%4 of the lanes L/4, L/4+4, L/4+8, L/4+12.  With lane s pointing at key
//     (s/4) and at d-offset 4*(s%4), lane L ends up with four keys of column d = L: two reads give the
//     eight keys of a fragment.
// Rows that do not exist (tail of the context or of the column list) re-load an existing row; their
// keys are masked, so only finiteness of the staged values matters.
// ---------------------------------------------------------------------------------------------
template <int D>
struct DirectCfg {
    static_assert(D == 128 || D == 64, "head dimension");
    static constexpr int RB = D * 2;                      // bytes per row
    static constexpr int DS = RB / 16;                    // 16-byte slots per row
    static constexpr int RPI = 64 / DS;                   // rows per transfer instruction
    static constexpr int NI = BN / RPI;                   // transfer instructions per operand tile
    static constexpr int IPW = NI / 4;                    // ... per wave
    static constexpr int K_ISTR = D == 128 ? 1088 : 1024; // LDS bytes from one K transfer to the next
    static constexpr int V_ISTR = 1024;
    static constexpr int K_BYTES = NI * K_ISTR, V_BYTES = NI * V_ISTR, TILE_BYTES = K_BYTES + V_BYTES;
    static constexpr int STEP = 4 * RPI * RB;             // global bytes between a wave's consecutive transfers
    static constexpr int KSTEPS = D / 16, DBLK = D / 32;
    static constexpr int KA = D == 128 ? 2 : 4;           // K fragment address registers
    // slot swizzles (XOR on the 16-byte slot index inside a row); both are unchanged by adding a
    // multiple of 16 (d = 128) or 32 (d = 64) to the row
    __device__ static constexpr int kswz(int row) { return D == 128 ? (row & 3) : (((row >> 1) & 3) | (((row >> 3) & 1) << 2)); }
    __device__ static constexpr int vswz(int row) { return D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2); }
};

// OBLDS: the head's diagonal bitmap is copied to LDS (short contexts); otherwise it is read from global
// memory where needed (the masks of a tile are computed one tile ahead, under the transfer wait), which
// keeps two workgroups per CU at long contexts.
template <int D, bool OBLDS>
__global__ __launch_bounds__(PREFILL_THREADS, 2) void prefill_bf16_kernel(PrefillArgs a) {
    using C = DirectCfg<D>;
    using T = bf16_t;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* tiles = smem;                                         // [2][TILE_BYTES]
    uint32_t* ob_lds = reinterpret_cast<uint32_t*>(smem + 2 * C::TILE_BYTES);
    int32_t* colring = reinterpret_cast<int32_t*>(ob_lds + (OBLDS ? a.words + 1 : 0));   // [3][64]
    int32_t* wcnt = colring + 192;                                       // [8]
    uint16_t* kbl = reinterpret_cast<uint16_t*>(wcnt + 8);               // [tab_len] active key blocks | flags << 14
    uint8_t* tab = reinterpret_cast<uint8_t*>(kbl + ((a.tab_len + 7) & ~7));   // [tab_len] this head's per-j table
    const uint32_t tiles_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)tiles;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r32 = lane & 31, g = lane >> 5;

    // ---- per-lane constants of the transfers: this lane fills slot sl of row rowlane (+ 4*RPI per
    // further instruction of the wave) and fetches the chunk the swizzle assigns to that slot
    const int rowlane = C::RPI * wv + lane / C::DS;
    const int sl = lane % C::DS;
    const uint32_t kcpart = 16u * (uint32_t)(sl ^ C::kswz(rowlane));
    const uint32_t vcpart = 16u * (uint32_t)(sl ^ C::vswz(rowlane));
    const uint32_t kvoff0 = (uint32_t)rowlane * C::RB + kcpart, vvoff0 = (uint32_t)rowlane * C::RB + vcpart;
    // ---- K fragment reads: row r32 (+32), chunk 2c+g sits in slot (2c+g) ^ kswz
    int kaddr[C::KA];
    {
        const int x = C::kswz(r32);
        const int krow = (r32 / C::RPI) * C::K_ISTR + (r32 % C::RPI) * C::RB;
#pragma unroll
        for (int j = 0; j < C::KA; ++j) kaddr[j] = krow + 32 * (j ^ (x >> 1)) + 16 * (g ^ (x & 1));
    }
    // ---- V^T fragment reads (see the header comment): key 4g + L16/4 (+8, +16 q4), 64-byte block i
    int vaddr[C::DBLK];
    {
        const int L16 = lane & 15, beta = (lane >> 4) & 1;
        const int lrow = 4 * g + (L16 >> 2);
        const int y = C::vswz(lrow) >> 2;
#pragma unroll
        for (int i = 0; i < C::DBLK; ++i) vaddr[i] = C::K_BYTES + lrow * C::RB + 64 * (i ^ y) + 32 * beta + 8 * (L16 & 3);
    }

    __shared__ int item_s;
  for (;;) {                                               // persistent: one (head, row block) item per trip
    __syncthreads();                                       // everyone is done with the previous item's LDS
    if (tid == 0) item_s = pop_item(a, blockIdx.x & 7);    // taken only when needed: items are coarse, reserving early hurts the tail
    __syncthreads();
    const int item = __builtin_amdgcn_readfirstlane(item_s);
    if (item < 0) break;
    const int bh = item >> 16, qb = item & 0xFFFF;
    const int b = bh / a.Hq, h = bh % a.Hq, kvh = h / a.G;
    const int64_t n = a.n, row0 = n - a.n_hat;
    const int64_t blockpos = a.pos0 + (int64_t)qb * BM;                  // multiple of 128
    const int64_t posmax = (blockpos + BM - 1 < n - 1) ? blockpos + BM - 1 : n - 1;
    const unsigned char* Kg = reinterpret_cast<const unsigned char*>(a.k) + ((int64_t)b * a.Hkv + kvh) * n * C::RB;
    const unsigned char* Vg = reinterpret_cast<const unsigned char*>(a.v) + ((int64_t)b * a.Hkv + kvh) * n * C::RB;
    const T* Qg = reinterpret_cast<const T*>(a.q) + (int64_t)bh * a.n_hat * D;
    const uint8_t* tabg = a.tab + (int64_t)bh * a.tab_len;

    const uint32_t* obg = a.obits + (int64_t)bh * (a.words + 1);          // zero word + bitmap of this head
    if (OBLDS) for (int i = tid; i < a.words + 1; i += PREFILL_THREADS) ob_lds[i] = obg[i];
    const uint32_t* ob = OBLDS ? ob_lds : obg;
    for (int i = tid; i < a.tab_len; i += PREFILL_THREADS) tab[i] = tabg[i];
    const int64_t pos = blockpos + 32 * wv + r32;
    const bool row_ok = (pos >= row0) && (pos < n);
    Frag<T> qf[C::KSTEPS];
    if (row_ok) {
        const T* qrow = Qg + (pos - row0) * D;
#pragma unroll
        for (int c = 0; c < C::KSTEPS; ++c) load_frag(qf[c], qrow + 16 * c + 8 * g);
    } else {
#pragma unroll
        for (int c = 0; c < C::KSTEPS; ++c) zero_frag(qf[c]);
    }
    const bool all_ok = __ballot(row_ok) == ~0ull;

    // ---- ordered list of the key blocks phase 1 visits (flags of the per-j table ride in bits 14-15)
    const int64_t jb = blockpos / BN;                      // even
    const int kb_hi = (int)(posmax / BN);
    int n1 = 0;
    for (int base = 0; base <= kb_hi; base += PREFILL_THREADS) {
        const int kb = base + tid;
        const uint8_t f = kb <= kb_hi ? tabg[jb - kb + 1] : (uint8_t)0;
        const bool act = f & 1;
        const uint64_t bal = __ballot(act);
        if (lane == 0) wcnt[wv] = __popcll(bal);
        __syncthreads();
        int off = n1;
        for (int w2 = 0; w2 < wv; ++w2) off += wcnt[w2];
        if (act) kbl[off + __popcll(bal & ((1ull << lane) - 1ull))] = (uint16_t)(kb | ((f & 2) << 13));
        n1 += wcnt[0] + wcnt[1] + wcnt[2] + wcnt[3];
        __syncthreads();
    }
    n1 = __builtin_amdgcn_readfirstlane(n1);
    int nv = a.v_cnt[bh]; if (nv > a.cap_v) nv = a.cap_v; if (nv < 0) nv = 0;
    const int32_t* vi = a.v_idx + (int64_t)bh * a.cap_v;
    if (a.hflag[bh] & 3) nv = 0;                           // every diagonal is selected (phase 1 covers all cells), or the list is unusable
    if (nv > 0 && (int64_t)vi[nv - 1] > posmax) {          // ascending list: binary search for the first column > posmax
        int lo = 0, hi = nv - 1;
        while (lo < hi) { const int mid = (lo + hi) >> 1; if ((int64_t)vi[mid] > posmax) hi = mid; else lo = mid + 1; }
        nv = lo;
    }
    const int n2 = (nv + BN - 1) / BN;
    const int ntiles = n1 + n2;

    f32x16 oacc[C::DBLK];
#pragma unroll
    for (int i = 0; i < C::DBLK; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;                  // m_run in raw logit units
    const float sc2 = a.scale_log2e;
    // The running reference m_run follows the row maximum lazily: it moves only when a tile exceeds it
    // by more than 2^8 in the exponent, so probabilities stay below 256 (exact in fp32 and bf16 alike)
    // and most tiles need no rescaling of the accumulators.
    const float lazy = 8.0f / sc2;

    // ---- staging.  Wave wv issues transfer instructions wv, wv+4, ... of each operand; instruction q
    // carries tile rows RPI*q .. RPI*q+RPI-1.  A row beyond the context re-loads the last row, a missing
    // column re-loads row 0: every slot is always written with finite data and needs no exec masking.
    // (Measured: spreading the transfers over the products of the previous tile instead of issuing
    // them together is slower; a transfer stalls the wave that issues it for as long as the vector
    // memory pipeline is busy, which then also stalls its matrix pipeline.)
    auto issue = [&](int t) {                              // global -> LDS buffer t & 1 for tile t
        const uint32_t dst = tiles_lds + (uint32_t)((t & 1) * C::TILE_BYTES);
        const uint32_t kdst = dst + (uint32_t)(wv * C::K_ISTR), vdst = dst + (uint32_t)(C::K_BYTES + wv * C::V_ISTR);
        if (t < n1) {
            const int64_t key0 = (int64_t)(__builtin_amdgcn_readfirstlane((int)kbl[t]) & 0x3FFF) * BN;
            const unsigned char* kb_ = Kg + key0 * C::RB;
            const unsigned char* vb_ = Vg + key0 * C::RB;
            if (key0 + BN <= n) {
#pragma unroll
                for (int i = 0; i < C::IPW; ++i) dma16(kb_ + i * C::STEP, kvoff0, kdst + (uint32_t)(4 * i * C::K_ISTR));
#pragma unroll
                for (int i = 0; i < C::IPW; ++i) dma16(vb_ + i * C::STEP, vvoff0, vdst + (uint32_t)(4 * i * C::V_ISTR));
            } else {                                       // last key block of the context: clamp the rows
                const int last = (int)(n - 1 - key0);
#pragma unroll
                for (int i = 0; i < C::IPW; ++i) {
                    const int row = rowlane + 4 * C::RPI * i;
                    const uint32_t ro = (uint32_t)(row <= last ? row : last) * C::RB;
                    dma16(kb_, ro + kcpart, kdst + (uint32_t)(4 * i * C::K_ISTR));
                    dma16(vb_, ro + vcpart, vdst + (uint32_t)(4 * i * C::V_ISTR));
                }
            }
        } else {
            const int32_t* cols = colring + (t % 3) * BN;
#pragma unroll
            for (int i = 0; i < C::IPW; ++i) {
                int32_t col = cols[rowlane + 4 * C::RPI * i];
                if (col < 0) col = 0;
                const uint32_t ro = (uint32_t)col * C::RB;
                dma16(Kg, ro + kcpart, kdst + (uint32_t)(4 * i * C::K_ISTR));
                dma16(Vg, ro + vcpart, vdst + (uint32_t)(4 * i * C::V_ISTR));
            }
        }
    };

    // One tile: S^T = K Q^T, online softmax, O^T += V^T P^T.  The products run in a pinned order
    // (a scheduling barrier after each) with the LDS fragment reads a fixed number of products ahead.
    auto process = [&](int tileoff, uint32_t am0, uint32_t am1, bool full) {
        const unsigned char* tile = tiles + tileoff;
        f32x16 s[2];
        bool act[2];
        act[0] = __ballot(am0 != 0u) != 0ull;
        act[1] = __ballot(am1 != 0u) != 0ull;
        if (!act[0] && !act[1]) return;                    // none of this wave's rows has an allowed cell here
        const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        s[0] = zero16; s[1] = zero16;
        constexpr int SUB = (32 / C::RPI) * C::K_ISTR;     // LDS bytes from key r to key r + 32
        const bool both = act[0] && act[1];
        if (both) {
            // 2 * KSTEPS products in a fixed order; K fragments are read RING_S products ahead of their use
            constexpr int NP = 2 * C::KSTEPS, R = LS_RING_S;
            Frag<T> kf[NP];
            auto kload = [&](int i) {
                const int c = i >> 1;
                load_frag(kf[i], tile + kaddr[c & (C::KA - 1)] + (i & 1) * SUB + 32 * (c & ~(C::KA - 1)));
            };
#pragma unroll
            for (int i = 0; i < R; ++i) kload(i);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                mma(s[i & 1], kf[i], qf[i >> 1]);          // s[r] = <k_{8(r/4)+4g+r%4}, q_row>
                if (i + R < NP) kload(i + R);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            // one 32-key half: KSTEPS products on one accumulator, same ring
            auto half = [&](auto subc) {
                constexpr int sub = decltype(subc)::value;
                constexpr int R = LS_RING_S < C::KSTEPS ? LS_RING_S : C::KSTEPS;
                Frag<T> kf[C::KSTEPS];
                auto kload = [&](int c) { load_frag(kf[c], tile + kaddr[c & (C::KA - 1)] + sub * SUB + 32 * (c & ~(C::KA - 1))); };
#pragma unroll
                for (int c = 0; c < R; ++c) kload(c);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int c = 0; c < C::KSTEPS; ++c) {
                    mma(s[sub], kf[c], qf[c]);
                    if (c + R < C::KSTEPS) kload(c + R);
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            if (act[0]) half(std::integral_constant<int, 0>{}); else half(std::integral_constant<int, 1>{});
        }
        float mx = -INFINITY;
        if (full) {
#pragma unroll
            for (int sub = 0; sub < 2; ++sub)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[sub][r]);
        } else {
#pragma unroll
            for (int sub = 0; sub < 2; ++sub) {
                const uint32_t amg = (sub ? am1 : am0) >> (4 * g);   // register r of this lane: key 8(r/4) + 4g + r%4
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float x = (amg & (1u << (8 * (r >> 2) + (r & 3)))) ? s[sub][r] : -INFINITY;
                    s[sub][r] = x;
                    mx = fmaxf(mx, x);
                }
            }
        }
        mx = fmaxf(mx, xor32(mx));
        const float m_new = (mx > m_run + lazy) ? mx : m_run;            // -inf + lazy = -inf: the first finite tile always moves it
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        const float corr = fast_exp2((m_run - m_safe) * sc2);
        const float mneg = -m_safe * sc2;
        m_run = m_new;
        float ps4[4] = {0.f, 0.f, 0.f, 0.f};               // four short add chains instead of one long one
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = fast_exp2(__builtin_fmaf(s[sub][r], sc2, mneg));
                s[sub][r] = p;
                ps4[r & 3] += p;
            }
        l_run = l_run * corr + ((ps4[0] + ps4[1]) + (ps4[2] + ps4[3]));
        if (__ballot(corr != 1.0f) != 0ull) {
#pragma unroll
            for (int i = 0; i < C::DBLK; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[i][r] *= corr;
        }
        auto vt_frag = [&](Frag<T>& vf, int q4, int i) {     // V^T fragment: keys 16*q4.., output block i
            const unsigned char* va = tile + vaddr[i] + 16 * q4 * C::RB;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(va));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(va + 8 * C::RB));
            struct U { s16x4 a, b; } u = {lo, hi};
            vf.v = __builtin_bit_cast(bf16x8, u);
        };
        // P*V: per 32-key half, 2 * DBLK products in a fixed order (16-key chunk q4, output block i); V^T
        // fragments are read RING_P products ahead
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            if (act[sub]) {
                constexpr int NPV = 2 * C::DBLK, R = LS_RING_P < NPV ? LS_RING_P : NPV;
                Frag<T> pf[2];
#pragma unroll
                for (int h2 = 0; h2 < 2; ++h2) {
                    float pv[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) pv[e] = s[sub][8 * h2 + e];
                    pack_frag(pf[h2], pv);
                }
                Frag<T> vf[NPV];
#pragma unroll
                for (int k = 0; k < R; ++k) vt_frag(vf[k], 2 * sub + k / C::DBLK, k % C::DBLK);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int k = 0; k < NPV; ++k) {
                    mma(oacc[k % C::DBLK], vf[k], pf[k / C::DBLK]);
                    if (k + R < NPV) vt_frag(vf[k + R], 2 * sub + (k + R) / C::DBLK, (k + R) % C::DBLK);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    };

    // cell masks of tile t for this lane's row: bit j of am0 / am1 = key j / 32 + j of the tile is allowed
    uint32_t am0 = 0u, am1 = 0u;
    bool full = false;
    auto masks = [&](int t) {
        am0 = 0u; am1 = 0u; full = false;
        if (t < n1) {
            const int e = __builtin_amdgcn_readfirstlane((int)kbl[t]);
            const int64_t key0 = (int64_t)(e & 0x3FFF) * BN;
            const bool fullflag = (e >> 14) & 1;
            if (!row_ok) { am0 = am1 = 0u; }
            else if (fullflag) { am0 = am1 = 0xFFFFFFFFu; }
            else {
                const int64_t d0 = pos - key0;             // diagonal of the tile's first key
                am0 = __brev(window32(ob, d0 - 31));
                am1 = __brev(window32(ob, d0 - 63));
            }
            full = fullflag && all_ok;
        } else {
            const int32_t* cols = colring + (t % 3) * BN;
            const int base = (t - n1) * BN;
            const int cnt = nv - base < BN ? nv - base : BN;
            const int32_t mycol = lane < cnt ? cols[lane] : 0;
            const uint8_t f = lane < cnt ? tab[jb - (mycol >> 6) + 1] : (uint8_t)3;
            const uint64_t drop = __ballot(f == 3);        // wholly covered by phase 1 (or no such slot)
            const uint64_t chk = __ballot(f == 1);         // partly covered: test cell by cell
            uint64_t am = 0ull;
            if (row_ok) {
                if ((int64_t)cols[cnt - 1] <= pos) am = cnt >= 64 ? ~0ull : ((1ull << cnt) - 1ull);
                else for (int i = 0; i < cnt; ++i) if ((int64_t)cols[i] <= pos) am |= 1ull << i;
                am &= ~drop;
                uint64_t todo = chk & am;
                while (todo) {
                    const int i = __ffsll((unsigned long long)todo) - 1;
                    todo &= todo - 1;
                    const int64_t o = pos - cols[i];       // >= 0 here
                    if ((ob[(o >> 5) + 1] >> (o & 31)) & 1u) am &= ~(1ull << i);   // cell already counted on its diagonal
                }
            }
            am0 = (uint32_t)am; am1 = (uint32_t)(am >> 32);
        }
    };

    // column ids of gathered tile t: fetched into a register one iteration before they are written to
    // LDS (slot t % 3), which happens one iteration before tile t is issued.  The global load is thus
    // never waited for while transfers are in flight.
    auto fetch_cols = [&](int t) -> int32_t {
        if (t >= n1 && t < ntiles && tid < BN) {
            const int idx = (t - n1) * BN + tid;
            return idx < nv ? vi[idx] : -1;
        }
        return -1;
    };
    auto store_cols = [&](int t, int32_t c) {
        if (t >= n1 && t < ntiles && tid < BN) colring[(t % 3) * BN + tid] = c;
    };

    store_cols(0, fetch_cols(0));
    store_cols(1, fetch_cols(1));
    int32_t colpre = fetch_cols(2);
    __syncthreads();                                       // bitmap, table, kbl, first column ids visible
    if (ntiles > 0) { issue(0); masks(0); }
    wait_transfers();
    __syncthreads();

    for (int t = 0; t < ntiles; ++t) {
        store_cols(t + 2, colpre);
        colpre = fetch_cols(t + 3);
        if (t + 1 < ntiles) issue(t + 1);
        process((t & 1) * C::TILE_BYTES, am0, am1, full);
        if (t + 1 < ntiles) masks(t + 1);                  // its LDS reads overlap the wait below
        wait_transfers();                                  // this wave's transfers of tile t+1 have landed
        __syncthreads();
    }

    const float l_tot = l_run + xor32(l_run);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    if (row_ok) {
        T* orow = reinterpret_cast<T*>(a.out) + ((int64_t)bh * a.n_hat + (pos - row0)) * D;
#pragma unroll
        for (int i = 0; i < C::DBLK; ++i)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                const int d0 = 32 * i + 8 * rq + 4 * g;
                store_out4(orow + d0, oacc[i][4 * rq] * inv, oacc[i][4 * rq + 1] * inv,
                           oacc[i][4 * rq + 2] * inv, oacc[i][4 * rq + 3] * inv);
            }
        if (a.lse && g == 0)
            a.lse[(int64_t)bh * a.n_hat + (pos - row0)] =
                l_tot > 0.f ? (m_run * sc2 + log2f(l_tot)) * 0.69314718055994531f : -INFINITY;
    }
  }                                                        // next item
}

template <int D>
static size_t prefill_bf16_smem(int words, int tab_len, bool oblds) {
    return 2 * (size_t)DirectCfg<D>::TILE_BYTES + (oblds ? (size_t)(words + 1) * 4 : 0) + 192 * 4 + 8 * 4 +
           (size_t)((tab_len + 7) & ~7) * 2 + (size_t)tab_len + 16;
}
// the bitmap goes to LDS when two workgroups still fit a CU's 160 KB with it
template <int D>
static bool prefill_bf16_oblds(int words, int tab_len) {
    return 2 * (prefill_bf16_smem<D>(words, tab_len, true) + 1024) <= 160 * 1024;
}

template <int D, bool OBLDS>
static hipError_t launch_prefill_bf16_t(const PrefillArgs& a, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
    const size_t smem = prefill_bf16_smem<D>(a.words, a.tab_len, OBLDS);
    // with events: they take the start and stop time stamps of this dispatch itself, no marker goes into the stream
    if (ev0 && ev1) hipExtLaunchKernelGGL((prefill_bf16_kernel<D, OBLDS>), dim3(persistent_grid(a)), dim3(PREFILL_THREADS), (uint32_t)smem, st, ev0, ev1, 0, a);
    else hipLaunchKernelGGL((prefill_bf16_kernel<D, OBLDS>), dim3(persistent_grid(a)), dim3(PREFILL_THREADS), smem, st, a);
    return hipGetLastError();
}
template <int D>
static hipError_t launch_prefill_bf16(const PrefillArgs& a, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
    return prefill_bf16_oblds<D>(a.words, a.tab_len) ? launch_prefill_bf16_t<D, true>(a, st, ev0, ev1) : launch_prefill_bf16_t<D, false>(a, st, ev0, ev1);
}

template <typename T, int D>
static size_t prefill_smem_t(int words, int tab_len) {
    using C = TileCfg<T, D>;
    return 2 * (size_t)C::K_BYTES + 2 * (size_t)C::VT_BYTES + (size_t)(words + 1) * 4 + 128 * 4 + 8 * 4 +
           (size_t)((tab_len + 7) & ~7) * 2 + (size_t)tab_len + 16;
}

template <typename T, int D>
static hipError_t launch_prefill_t(const PrefillArgs& a, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
    const size_t smem = prefill_smem_t<T, D>(a.words, a.tab_len);
    if (ev0 && ev1) hipExtLaunchKernelGGL((prefill_kernel<T, D>), dim3(persistent_grid(a)), dim3(PREFILL_THREADS), (uint32_t)smem, st, ev0, ev1, 0, a);
    else hipLaunchKernelGGL((prefill_kernel<T, D>), dim3(persistent_grid(a)), dim3(PREFILL_THREADS), smem, st, a);
    return hipGetLastError();
}

hipError_t init_prefill_kernels() {
    hipError_t e;
    if ((e = allow_full_lds(&prefill_bf16_kernel<128, true>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&prefill_bf16_kernel<128, false>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&prefill_bf16_kernel<64, true>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&prefill_bf16_kernel<64, false>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&prefill_kernel<float, 128>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&prefill_kernel<float, 64>)) != hipSuccess) return e;
    return allow_full_lds(&plan_kernel);
}

size_t prefill_smem_bytes(int dtype, int d, int words, int tab_len) {
    if (dtype == 0 && d == 128) return prefill_bf16_smem<128>(words, tab_len, prefill_bf16_oblds<128>(words, tab_len));
    if (dtype == 0 && d == 64) return prefill_bf16_smem<64>(words, tab_len, prefill_bf16_oblds<64>(words, tab_len));
    if (dtype == 1 && d == 128) return prefill_smem_t<float, 128>(words, tab_len);
    return prefill_smem_t<float, 64>(words, tab_len);
}

hipError_t launch_plan(const PlanArgs& a, int BH, hipStream_t st) {
    const size_t smem = (size_t)a.words * 4;
    hipLaunchKernelGGL(plan_kernel, dim3(BH), dim3(1024), smem, st, a);
    return hipGetLastError();
}

int prefill_block_rows() { return BM; }

hipError_t launch_sched(const SchedArgs& a, hipStream_t st) {
    hipLaunchKernelGGL(sched_kernel, dim3(8), dim3(SCHED_THREADS), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_prefill(const PrefillArgs& a, int dtype, int d, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
    if (dtype == 0 && d == 128) return launch_prefill_bf16<128>(a, st, ev0, ev1);
    if (dtype == 0 && d == 64) return launch_prefill_bf16<64>(a, st, ev0, ev1);
    if (dtype == 1 && d == 128) return launch_prefill_t<float, 128>(a, st, ev0, ev1);
    if (dtype == 1 && d == 64) return launch_prefill_t<float, 64>(a, st, ev0, ev1);
    return hipErrorInvalidValue;
}

}  // namespace ls
