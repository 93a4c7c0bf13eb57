// Per-head line selection (Alg. 2 from Desc_Sort on) and top-B retention (Alg. 3), gfx950.
//
//   sort_seg_kernel / sort_merge_kernel
//                 Desc_Sort: the n line weights of a list in descending order, equal weights in
//                 ascending index order.  Segments of 2048 to 8192 elements are sorted inside LDS by a stable
//                 LSD radix sort (4 x 8 bits): each of the 16 waves owns a contiguous slice, counts its
//                 digits in its own histogram, and scatters its slice in order (ranks among equal
//                 digits from wave ballots and the wave's running counters; no atomics decide an
//                 output position).  The sorted segments are then merged by rank: every element's
//                 final position is its position in its segment plus, by bisection, the number of
//                 elements of the other segments that precede it.
//   walk_kernel   one workgroup of six waves per head: the greedy loop of Alg. 2 in binary32 with the operands
//                 and operation order of the definition.  One wave decides runs of up to 512 picks from one
//                 list with its lanes, one accumulates the running sum pick by pick behind it and finds
//                 the pick that reaches the target, and two waves per list stage the sorted list and its
//                 overlap prefix sums in LDS ahead of both.
//   emit_kernel   one workgroup per (head, list): the chosen prefix of a sorted list becomes an
//                 ascending index list (bitmap in LDS + prefix popcount).
//   topb_*        Alg. 3: the `budget` largest scores per KV head by a three-digit radix select on the
//                 float bit patterns, ties broken towards smaller indices, ascending output; a head's
//                 scores are spread over many workgroups, one launch per step.
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

constexpr int WALK_BLK = 1024;                 // entries of a sorted list the walk stages at a time
static_assert(WALK_BLK == SELECT_HEAD_LINES, "the merge writes the walk's first block in order");
constexpr int SORT_THREADS = 1024;
constexpr int SORT_WAVES = 16;
constexpr int SORT_SEG_MAX = 8192;             // most elements one workgroup sorts inside LDS
constexpr int SORT_SEG_MIN = 2048;
constexpr size_t sort_lds_bytes(int seg) { return (size_t)2 * seg * 4 + (size_t)2 * seg * 2 + SORT_WAVES * 256 * 4 + 256 * 4; }

// grid (segments, 2, BH): list 0 = diagonals (slash), 1 = columns (vert).  Sorts elements
// [seg * SEG, +SEG) of one list entirely in LDS and writes the sorted keys (skey0) and their
// line indices (sidx0) back to the same range.
template <int SEG>
__global__ __launch_bounds__(SORT_THREADS) void sort_seg_kernel(SelectArgs a) {
    constexpr int SLICE = SEG / SORT_WAVES;
    extern __shared__ __align__(16) unsigned char sort_lds[];
    uint32_t* kb0 = reinterpret_cast<uint32_t*>(sort_lds);
    uint32_t* kb1 = kb0 + SEG;
    uint16_t* ib0 = reinterpret_cast<uint16_t*>(kb1 + SEG);
    uint16_t* ib1 = ib0 + SEG;
    uint32_t (*hist)[256] = reinterpret_cast<uint32_t (*)[256]>(ib1 + SEG);
    uint32_t* dbase = &hist[SORT_WAVES][0];
    const int seg = blockIdx.x, list = blockIdx.y, bh = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int64_t n = a.n;
    const int64_t base0 = (int64_t)seg * SEG;
    const int cnt = (int)(n - base0 < SEG ? n - base0 : SEG);
    const float* src = (list == 0 ? a.slash : a.vert) + (int64_t)bh * n + base0;
    const int64_t out0 = ((int64_t)list * a.BH + bh) * n + base0;
    // slots past the end of the list hold the largest key: they sort behind every element and, being
    // the highest local indices, turn behind equal keys as well
    for (int i = tid; i < SEG; i += SORT_THREADS) {
        kb0[i] = i < cnt ? desc_key(src[i]) : 0xFFFFFFFFu;
        ib0[i] = (uint16_t)i;
    }
    const int lo = wv * SLICE;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 8 * pass;
        const uint32_t* kin = (pass & 1) ? kb1 : kb0;
        const uint16_t* iin = (pass & 1) ? ib1 : ib0;
        uint32_t* kout = (pass & 1) ? kb0 : kb1;
        uint16_t* iout = (pass & 1) ? ib0 : ib1;
        for (int i = tid; i < SORT_WAVES * 256; i += SORT_THREADS) (&hist[0][0])[i] = 0u;
        __syncthreads();
        // this wave's slice, read once per pass and ahead of the counting (the compiler does not move reads across atomics)
        uint32_t keys[SLICE / 64]; uint16_t idxs[SLICE / 64];
#pragma unroll
        for (int c = 0; c < SLICE / 64; ++c) { keys[c] = kin[lo + 64 * c + lane]; idxs[c] = iin[lo + 64 * c + lane]; }
        if (pass < 3) {
#pragma unroll
            for (int c = 0; c < SLICE / 64; ++c) atomicAdd(&hist[wv][(keys[c] >> shift) & 255u], 1u);
        } else {
            // the top byte (sign and upper exponent bits) takes few values, and 64 atomics on one counter take turns:
            // three times over, the lanes that share the digit of the first lane not yet counted add once together;
            // what is left adds one by one
#pragma unroll
            for (int c = 0; c < SLICE / 64; ++c) {
                const uint32_t dg = keys[c] >> 24;
                uint64_t todo = ~0ull;
#pragma unroll
                for (int round = 0; round < 3; ++round) {
                    if (todo == 0ull) break;
                    const int first = __ffsll((unsigned long long)todo) - 1;
                    const uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane((int)dg, first);
                    const uint64_t same = __ballot(dg == d0) & todo;
                    if (lane == first) atomicAdd(&hist[wv][d0], (uint32_t)__popcll(same));
                    todo &= ~same;
                }
                if ((todo >> lane) & 1ull) atomicAdd(&hist[wv][dg], 1u);
            }
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
            uint32_t v[4], sm = 0;
#pragma unroll
            for (int q = 0; q < 4; ++q) { v[q] = dbase[4 * tid + q]; sm += v[q]; }
            uint32_t inc = sm;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) { const uint32_t t = __shfl_up(inc, off, 64); if (lane >= off) inc += t; }
            uint32_t ex = inc - sm;
#pragma unroll
            for (int q = 0; q < 4; ++q) { dbase[4 * tid + q] = ex; ex += v[q]; }
        }
        __syncthreads();
        if (tid < 256) {
            const uint32_t bs = dbase[tid];
            for (int w = 0; w < SORT_WAVES; ++w) hist[w][tid] += bs;
        }
        __syncthreads();
        // in-order scatter of this wave's slice: inside a 64-element chunk the rank among equal digits
        // comes from wave ballots, across chunks from the wave's running counters
        // (the wave's counters are read and written with relaxed atomics: plain LDS accesses that the compiler keeps
        // in program order around the wave barriers; a volatile pointer would turn them into flat accesses)
        uint32_t* myh = hist[wv];
#pragma unroll
        for (int c = 0; c < SLICE / 64; ++c) {
            const uint32_t key = keys[c];
            const uint16_t idx = idxs[c];
            const uint32_t dg = (key >> shift) & 255u;
            // lanes whose digit differs from mine in some bit: bit b of the lanes' digits as a wave mask, against
            // my own bit b spread over a word
            uint32_t diff_lo = 0u, diff_hi = 0u;
#pragma unroll
            for (int bit = 0; bit < 8; ++bit) {
                const int32_t m = (int32_t)(dg << (31 - bit)) >> 31;               // 0 or ~0
                const uint64_t bal = __ballot(m != 0);
                diff_lo |= (uint32_t)bal ^ (uint32_t)m;
                diff_hi |= (uint32_t)(bal >> 32) ^ (uint32_t)m;
            }
            const uint64_t peers = ~(((uint64_t)diff_hi << 32) | diff_lo);
            const uint64_t below = peers & ((1ull << lane) - 1ull);
            const uint32_t rank = __popcll(below);
            const uint32_t pos = __atomic_load_n(&myh[dg], __ATOMIC_RELAXED) + rank;
            __builtin_amdgcn_wave_barrier();
            kout[pos] = key;
            iout[pos] = idx;
            if (below == 0ull) __atomic_store_n(&myh[dg], pos + (uint32_t)__popcll(peers), __ATOMIC_RELAXED);
            __builtin_amdgcn_wave_barrier();
        }
        __syncthreads();                                   // every wave is done with the counters and the input buffer
    }
    // four passes: the result sits in buffer 0
    for (int i = tid; i < cnt; i += SORT_THREADS) {
        a.skey0[out0 + i] = kb0[i];
        a.sidx0[out0 + i] = (int32_t)(base0 + ib0[i]);
    }
}

// grid (segments, 2, BH).  Final position of an element of segment q = its position inside q + the
// number of elements of every other segment that go before it: smaller key, or equal key in a segment
// of smaller line indices (the order stays stable).  The other segments' sorted keys are staged in
// LDS one at a time (two buffers: the next segment is loaded while the current one is searched) and
// searched by bisection.  Writes the line indices in sorted order (sidx1): a scattered store per line, which is
// why the weights and maxima are not written beside them; the walk fetches those through the indices, and only
// for the part of the order it gets to.
// Dynamic LDS: 2 * SEG keys.
template <int SEG>
__global__ __launch_bounds__(SORT_THREADS) void sort_merge_kernel(SelectArgs a) {
    constexpr int PER = SEG / SORT_THREADS;
    extern __shared__ __align__(16) unsigned char merge_lds[];
    uint32_t (*other)[SEG] = reinterpret_cast<uint32_t (*)[SEG]>(merge_lds);
    const int seg = blockIdx.x, list = blockIdx.y, bh = blockIdx.z;
    const int tid = threadIdx.x;
    const int64_t n = a.n;
    const int nseg = (int)((n + SEG - 1) / SEG);
    const int64_t lbase = ((int64_t)list * a.BH + bh) * n;
    const int64_t base0 = (int64_t)seg * SEG;
    const int cnt = (int)(n - base0 < SEG ? n - base0 : SEG);
    uint32_t key[PER], rank[PER], nxt[PER];
    auto fetch = [&](int q) {                               // keys of segment q, padded with the largest key
        const int64_t qb = (int64_t)q * SEG;
        const int qc = (int)(n - qb < SEG ? n - qb : SEG);
#pragma unroll
        for (int j = 0; j < PER; ++j) {
            const int i = tid + j * SORT_THREADS;
            nxt[j] = i < qc ? a.skey0[lbase + qb + i] : 0xFFFFFFFFu;
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int j = 0; j < PER; ++j) other[buf][tid + j * SORT_THREADS] = nxt[j];
    };
    int q = seg == 0 ? 1 : 0;
    if (q < nseg) fetch(q);
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int p = tid + j * SORT_THREADS;
        key[j] = p < cnt ? a.skey0[lbase + base0 + p] : 0xFFFFFFFFu;
        rank[j] = (uint32_t)p;
    }
    if (q < nseg) stage(0);
    __syncthreads();
    int buf = 0;
    while (q < nseg) {
        const int q2 = q + 1 == seg ? q + 2 : q + 1;
        if (q2 < nseg) fetch(q2);
        const int64_t qb = (int64_t)q * SEG;
        const int qc = (int)(n - qb < SEG ? n - qb : SEG);
        // number of i in [0, qc) with other[i] before key: other[i] < key, or <= key when the other segment is an
        // earlier one (its equal keys go first).  The segment is padded to its full power-of-two length with the
        // largest key, so the search has a fixed number of steps and the PER searches of a thread advance together:
        // their LDS reads are in flight at the same time (plain 32-bit compares: a 64-bit "key + 1" compare made the
        // compiler funnel all reads through one register pair, one wait each).
        // (positions are kept as LDS byte addresses: a probe then needs no address arithmetic beyond the
        // instruction's own offset)
        typedef const __attribute__((address_space(3))) uint32_t* lds_u32;
        const uint32_t base = (uint32_t)(uintptr_t)(lds_u32)other[buf];
        uint32_t la[PER];
#pragma unroll
        for (int j = 0; j < PER; ++j) la[j] = base;
        auto search = [&](auto earlier) {
            constexpr bool le = decltype(earlier)::value;
#pragma unroll
            for (int step = SEG / 2; step >= 1; step >>= 1) {
                uint32_t o[PER];
#pragma unroll
                for (int j = 0; j < PER; ++j) o[j] = *(lds_u32)(uintptr_t)(la[j] + 4u * (uint32_t)(step - 1));
#pragma unroll
                for (int j = 0; j < PER; ++j) if (le ? o[j] <= key[j] : o[j] < key[j]) la[j] += 4u * (uint32_t)step;
            }
            uint32_t o[PER];
#pragma unroll
            for (int j = 0; j < PER; ++j) o[j] = *(lds_u32)(uintptr_t)la[j];
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                const int r = (int)((la[j] - base) >> 2) + ((le ? o[j] <= key[j] : o[j] < key[j]) ? 1 : 0);
                rank[j] += (uint32_t)(r < qc ? r : qc);
            }
        };
        if (q < seg) search(std::true_type{}); else search(std::false_type{});
        if (q2 < nseg) stage(buf ^ 1);
        __syncthreads();                                   // this buffer is free again, the other one is filled
        buf ^= 1;
        q = q2;
    }
    // (the first WALK_BLK lines of the order also get their weight and maximum written, so that the walk can start
    // without a second round trip through the indices)
    const float* mx = (list == 0 ? a.smax : a.vmax) + (int64_t)bh * n;
    float* hw = a.head_w + ((int64_t)list * a.BH + bh) * WALK_BLK;
    float* hm = a.head_m + ((int64_t)list * a.BH + bh) * WALK_BLK;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int p = tid + j * SORT_THREADS;
        if (p < cnt) {
            const int32_t idx = a.sidx0[lbase + base0 + p];
            a.sidx1[lbase + rank[j]] = idx;
            if (rank[j] < (uint32_t)WALK_BLK) { hw[rank[j]] = key_to_float(key[j]); hm[rank[j]] = mx[idx]; }
        }
    }
}

// ---- the greedy loop ----------------------------------------------------------------------------
// One workgroup of six waves per head.  The loop of Alg. 2 is sequential, but three things about it are not:
//   * ol_s after k slashes were taken is the left-to-right binary32 sum of the first k maxima of
//     the slash list, whatever the interleaving with verticals was (likewise ol_v), so both
//     running overlaps are prefix arrays that can be filled ahead of the walk (still added one
//     element after the other, so every value is the one the sequential loop would hold);
//   * while the walk keeps taking from one list, the state of the other list is frozen, so the
//     next 64 ratio tests can be evaluated by the 64 lanes at once; a ballot gives the length of
//     the run of equal decisions.
//   * which list the next pick comes from does not depend on `sum`; only the end of the walk does.  So the
//     decisions can run ahead of the sum: they are handed over run by run (the gain of every pick, in pick
//     order) through a small ring in LDS, and whatever was decided beyond the pick that reaches the target
//     is dropped.
// What stays sequential are two chains of binary32 additions, one add per line each: the overlap prefix sums
// and `sum` with its exit test after every pick.  Both are evaluated by a wave whose lanes hold consecutive
// entries and pass the last partial sum to the right neighbour, one lane settling per pass, so every value is
// the one the sequential loop would hold and each pick sees exactly the operands, operation order and
// roundings of the definition.
constexpr int WALK_THREADS = 384;              // wave 0 decides the runs, wave 2 sums them; per list, waves 1 / 3 stage its
                                               // weights and lengths and waves 4 / 5 its overlap prefix sums
constexpr int WALK_E = 8;                      // consecutive list entries a lane looks at: a run has up to 64 * E picks
constexpr int WALK_RUN = 64 * WALK_E;
constexpr int WALK_NBLK = 4;                   // blocks of a list resident in LDS (a ring over sorted positions)
constexpr int WALK_CAP = WALK_BLK * WALK_NBLK;
constexpr int WALK_EB = WALK_BLK / 64;         // entries per lane when a block's prefix sums are added
static_assert(WALK_EB % 2 == 0 && WALK_RUN <= WALK_BLK, "a run never reaches beyond the block after the head's");

// The resident part of one sorted list, indexed by sorted position modulo WALK_CAP: weights, line lengths, and
// pre[p] = the overlap sum when the first p lines of the list have been taken.
struct WalkList { float cw[WALK_CAP], cl[WALK_CAP], pre[WALK_CAP]; };
// One run of picks from one list: the gain of each pick, how many of them count, and whether the walk ends
// after them because no line is left that adds anything.
struct WalkRun { float g[WALK_RUN]; int which, limit, last, pad; };
struct WalkSync { int staged[2], summed_blk[2], cur[2], summed, stop, done, err, runs, decided; float tot[2]; };
static_assert(offsetof(WalkSync, summed) % 8 == 0 && offsetof(WalkSync, stop) == offsetof(WalkSync, summed) + 4, "summed and stop are read as one 8-byte word");   // tot: a list's whole overlap sum
constexpr int WALK_RING = 4;                   // runs decided ahead of the running sum
constexpr size_t WALK_LDS_BYTES = 2 * sizeof(WalkList) + WALK_RING * sizeof(WalkRun) + sizeof(WalkSync);

__device__ __forceinline__ int walk_ld(const int* p) { return __builtin_amdgcn_readfirstlane(__atomic_load_n(p, __ATOMIC_RELAXED)); }
__device__ __forceinline__ void walk_st(int* p, int v) { __atomic_store_n(p, v, __ATOMIC_RELAXED); }

// Lane j holds the maxima m[0 .. E) of the list entries p0 + E j .. p0 + E j + E - 1.  Writes pre[i] = acc + (the
// maxima of the entries before entry i of the block, added left to right in binary32) for the 64 E entries of
// the block, pre pointing at the block's first entry, and returns the sum behind the last entry.  E is even.
template <int E>
__device__ __forceinline__ float walk_scan(const float (&m)[E], float* pre, float acc, int lane) {
    float x[E];
    // lane 0 has no left neighbour: the shift hands it 0, and its first addend is acc + m[0], so it holds exactly that
    const float addend0 = lane == 0 ? __fadd_rn(acc, m[0]) : m[0];
#pragma unroll
    for (int e = 0; e < E; ++e) x[e] = 0.f;
    for (int p = 0; p < 64; p += 2) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const float left = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(
                0, __builtin_bit_cast(int, x[E - 1]), 0x138 /* wave_shr:1 */, 0xF, 0xF, true));
            x[0] = __fadd_rn(left, addend0);
#pragma unroll
            for (int e = 1; e < E; ++e) x[e] = __fadd_rn(x[e - 1], m[e]);
        }
    }
    const float left = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(
        0, __builtin_bit_cast(int, x[E - 1]), 0x138 /* wave_shr:1 */, 0xF, 0xF, true));
    float2* dst = reinterpret_cast<float2*>(pre + E * lane);
    dst[0] = make_float2(lane == 0 ? acc : left, x[0]);
#pragma unroll
    for (int e = 2; e < E; e += 2) dst[e / 2] = make_float2(x[e - 1], x[e]);
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x[E - 1]), 63));
}

// ix[e] = the line at sorted position pos + e (the last line's index past the end of the list)
template <int E>
__device__ __forceinline__ void walk_indices(const int32_t* i_l, int pos, int n, int32_t (&ix)[E]) {
    typedef __attribute__((ext_vector_type(4))) int32_t i32x4;
    // (a wave-uniform choice: the list starts on a 16-byte boundary and the wave's last entry is inside it)
    const bool whole = (reinterpret_cast<uintptr_t>(i_l) & 15) == 0 && (pos & 3) == 0 &&
                       __builtin_amdgcn_readfirstlane(pos) + 64 * E <= n;
    if (E % 4 == 0 && whole) {
#pragma unroll
        for (int e = 0; e < E; e += 4) {
            const i32x4 v = *reinterpret_cast<const i32x4*>(i_l + pos + e);
            ix[e] = v.x; ix[e + 1] = v.y; ix[e + 2] = v.z; ix[e + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int e = 0; e < E; ++e) { const int i = pos + e; ix[e] = i_l[i < n ? i : n - 1]; }
    }
}
// m[e] = the largest entry of line ix[e], the line at sorted position pos + e (0 past the end of the list)
template <int E>
__device__ __forceinline__ void walk_maxima(const float* m_l, const int32_t (&ix)[E], int pos, int n, float (&m)[E]) {
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const float t = m_l[ix[e]];
        m[e] = pos + e < n ? t : 0.f;
    }
}

// Position of the first entry for which `p` holds, in the order entry 0 of lane 0, entry 1 of lane 0, ..., entry 0
// of lane 1, ... (WALK_RUN if it holds nowhere): every lane finds its own first entry, one ballot finds the lane.
__device__ __forceinline__ int walk_first(const bool (&p)[WALK_E]) {
    int fe = WALK_E;
#pragma unroll
    for (int e = WALK_E - 1; e >= 0; --e) fe = p[e] ? e : fe;
    const uint64_t any = __ballot(fe < WALK_E);
    if (any == 0ull) return WALK_RUN;
    const int l = __ffsll((unsigned long long)any) - 1;
    return WALK_E * l + __builtin_amdgcn_readlane(fe, l);
}

// grid (BH).  Reads the sorted lists (weights, maxima, indices) and writes taken counts.
//
// The waves share only LDS.  Each list is staged in blocks of WALK_BLK sorted positions into a ring of WALK_NBLK
// blocks: waves 1 / 3 write the weights and line lengths of a block (staged[l] = blocks written), waves 4 / 5
// its overlap prefix sums, reading the maxima straight from global memory (summed_blk[l]); both load the next
// block while they work on the current one.  Block b may be written once the deciding wave's head of that list
// has reached block b - WALK_NBLK + 1 (cur[l] = the head's block): nothing before the head is read again.  The
// deciding wave (0) needs the head's block and the one after it; it publishes cur[l] and runs = the number of
// runs it has put into the ring of runs; the summing wave (2) publishes summed = the number of runs it has
// taken out, and stop when the walk is over.  The summing wave writes the result; the deciding wave ends the
// stagers through `done`.  Every wait is a bounded spin that also ends when another wave has reported a failed
// wait, so all six waves leave in every case.
__global__ __launch_bounds__(WALK_THREADS) void walk_kernel(SelectArgs a) {
    extern __shared__ __align__(16) unsigned char walk_lds[];
    WalkList* lists = reinterpret_cast<WalkList*>(walk_lds);
    WalkRun* ring = reinterpret_cast<WalkRun*>(walk_lds + 2 * sizeof(WalkList));
    WalkSync* sync = reinterpret_cast<WalkSync*>(walk_lds + 2 * sizeof(WalkList) + WALK_RING * sizeof(WalkRun));
    const int bh = blockIdx.x, lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = (int)a.n;
    const int nblk = (n + WALK_BLK - 1) / WALK_BLK;
    const int64_t nh = a.n_hat;
    const int spin_limit = a.spin_limit;       // bound of every wait between the waves
    const int64_t seg_s = ((int64_t)0 * a.BH + bh) * a.n, seg_v = ((int64_t)1 * a.BH + bh) * a.n;

    if (threadIdx.x == 0) {
        sync->staged[0] = sync->staged[1] = 0; sync->summed_blk[0] = sync->summed_blk[1] = 0;
        sync->cur[0] = sync->cur[1] = 0; sync->done = 0; sync->err = 0;
        sync->runs = 0; sync->summed = 0; sync->decided = 0; sync->stop = 0;
    }
    __syncthreads();

    if (wv == 1 || wv == 3) {
        // ------------------------------------------------------------------ weights and lengths of one list
        const int l = wv == 1 ? 0 : 1;
        WalkList& L = lists[l];
        const int64_t seg = l == 0 ? seg_s : seg_v;
        const float* w_l = (l == 0 ? a.slash : a.vert) + (int64_t)bh * a.n;   // weights by line index
        const int32_t* i_l = a.sidx1 + seg;
        const int nh32 = (int)nh;
        constexpr int PER = WALK_BLK / 64;
        // the block after the last one written to LDS (indices and weights), and the indices of the one after it:
        // the weights are fetched through the indices, so the indices are requested a block earlier
        float fw[PER]; int32_t fx[PER], fxn[PER];
        auto fetch_idx = [&](int b, int32_t (&x)[PER]) {
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                const int gi = b * WALK_BLK + lane + j * 64;
                x[j] = i_l[gi < n ? gi : n - 1];
            }
        };
        auto fetch = [&](int b) {                          // fx <- fxn (block b), its weights, and block b + 1's indices
#pragma unroll
            for (int j = 0; j < PER; ++j) { fx[j] = fxn[j]; fw[j] = w_l[fx[j]]; }
            fetch_idx(b + 1, fxn);
        };
        {                                                  // block 0: its weights were written in order by the merge
            const float* hw = a.head_w + ((int64_t)l * a.BH + bh) * WALK_BLK;
            fetch_idx(0, fx);
#pragma unroll
            for (int j = 0; j < PER; ++j) { const int gi = lane + j * 64; fw[j] = hw[gi < n ? gi : n - 1]; }
            fetch_idx(1, fxn);
        }
        int b = 0;
        int spins = 0;
        while (walk_ld(&sync->done) == 0 && b < nblk) {
            if (b > walk_ld(&sync->cur[l]) + WALK_NBLK - 1) {
                __builtin_amdgcn_s_sleep(2);
                if (++spins > spin_limit) { walk_st(&sync->err, 1); break; }
                continue;
            }
            spins = 0;
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            const int slot = (b & (WALK_NBLK - 1)) * WALK_BLK;
#pragma unroll
            for (int j = 0; j < PER; ++j) {
                const int i = lane + j * 64;
                const bool in = b * WALK_BLK + i < n;
                const int len = n - fx[j] < nh32 ? n - fx[j] : nh32;       // line length in the n_hat x n block
                L.cw[slot + i] = in ? fw[j] : 0.f;
                L.cl[slot + i] = in ? (float)len : 1.f;
            }
            fetch(b + 1);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_wave_barrier();
            ++b;
            if (lane == 0) walk_st(&sync->staged[l], b);
        }
        return;
    }

    if (wv == 4 || wv == 5) {
        // ------------------------------------------------------------------ overlap prefix sums of one list
        // One add after the other, in list order.  Lane j owns E consecutive entries; a pass is "take the last sum
        // of the lane to the left, add my E maxima one after the other", and pass p settles lane p, so 64 passes
        // leave every lane with the sums the sequential loop would hold (the lanes to the right of the settled
        // ones compute values that the later passes replace).
        const int l = wv - 4;
        WalkList& L = lists[l];
        const int32_t* i_l = a.sidx1 + (l == 0 ? seg_s : seg_v);
        const float* m_l = (l == 0 ? a.smax : a.vmax) + (int64_t)bh * a.n;     // maxima by line index
        float m[WALK_EB], mn[WALK_EB];
        int32_t ix[WALK_EB];                   // line indices of the block after the next one's maxima
        {                                      // block 0: its maxima were written in order by the merge
            const float* hm = a.head_m + ((int64_t)l * a.BH + bh) * WALK_BLK;
#pragma unroll
            for (int e = 0; e < WALK_EB; ++e) { const int i = WALK_EB * lane + e; const float t = hm[i < n ? i : n - 1]; m[e] = i < n ? t : 0.f; }
        }
        walk_indices<WALK_EB>(i_l, WALK_BLK + WALK_EB * lane, n, ix);
        float acc = 0.f;                       // overlap sum behind the last entry summed so far
        int b = 0;
        int spins = 0;
        while (walk_ld(&sync->done) == 0 && b < nblk) {
            if (b > walk_ld(&sync->cur[l]) + WALK_NBLK - 1) {
                __builtin_amdgcn_s_sleep(2);
                if (++spins > spin_limit) { walk_st(&sync->err, 1); break; }
                continue;
            }
            spins = 0;
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            walk_maxima<WALK_EB>(m_l, ix, (b + 1) * WALK_BLK + WALK_EB * lane, n, mn);
            walk_indices<WALK_EB>(i_l, (b + 2) * WALK_BLK + WALK_EB * lane, n, ix);
            acc = walk_scan<WALK_EB>(m, L.pre + (b & (WALK_NBLK - 1)) * WALK_BLK, acc, lane);
#pragma unroll
            for (int e = 0; e < WALK_EB; ++e) m[e] = mn[e];
            if (b == nblk - 1 && lane == 0) sync->tot[l] = acc;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_wave_barrier();
            ++b;
            if (lane == 0) walk_st(&sync->summed_blk[l], b);
        }
        return;
    }

    if (wv == 2) {
        // ------------------------------------------------------------------ the running sum
        // Takes the runs in the order they were decided and adds their gains pick by pick; the first pick whose
        // sum reaches the target ends the walk.
        const float target = a.alpha * a.total[bh];
        float sum = 0.f;
        int cnt_s = 0, cnt_v = 0;              // lines taken from each list
        int k = 0;                             // runs summed
        bool failed = false, all = false;
        while (sum < target) {
            bool have = false;
            int spins = 0;
            for (;;) {
                if (walk_ld(&sync->runs) > k) { have = true; break; }
                if (walk_ld(&sync->decided)) {                       // stored after the last run was published
                    have = walk_ld(&sync->runs) > k;
                    failed = !have && walk_ld(&sync->err) != 0;
                    break;
                }
                if (++spins > spin_limit || walk_ld(&sync->err)) { failed = true; break; }
                __builtin_amdgcn_s_sleep(1);
            }
            if (!have) break;                  // both lists were used up (or a wait ran into its bound)
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            const WalkRun& R = ring[k & (WALK_RING - 1)];
            const int which = __builtin_amdgcn_readfirstlane(R.which);
            const int limit = __builtin_amdgcn_readfirstlane(R.limit);
            const int last = __builtin_amdgcn_readfirstlane(R.last);
            float g[WALK_E], x[WALK_E];
#pragma unroll
            for (int e = 0; e < WALK_E; e += 2) {
                const float2 t = *reinterpret_cast<const float2*>(&R.g[WALK_E * lane + e]);
                g[e] = t.x; g[e + 1] = t.y;
            }
            // Lane j ends up with the running sums after its E picks: x[0] = (x[E-1] of lane j-1) + g[0], x[e] =
            // x[e-1] + g[e], lane 0 starting from `sum`.  One pass of "take the left neighbour's last sum, add my
            // gains one after the other" over all lanes settles one more lane, in order, so ceil(limit / E) passes
            // reproduce the pick-by-pick additions exactly; the first entry whose sum reaches the target is the
            // pick the loop of the definition stops after.  (Lane 0 has no left neighbour: the shift hands it 0 and
            // its first addend is sum + g[0], so it holds exactly that.)
            const float addend0 = lane == 0 ? __fadd_rn(sum, g[0]) : g[0];
#pragma unroll
            for (int e = 0; e < WALK_E; ++e) x[e] = 0.f;
            for (int p0 = 0; p0 < limit; p0 += 4 * WALK_E) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float left = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(
                        0, __builtin_bit_cast(int, x[WALK_E - 1]), 0x138 /* wave_shr:1 */, 0xF, 0xF, true));
                    x[0] = __fadd_rn(left, addend0);
#pragma unroll
                    for (int e = 1; e < WALK_E; ++e) x[e] = __fadd_rn(x[e - 1], g[e]);
                }
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");         // the slot may be written again
            ++k;
            if (lane == 0) walk_st(&sync->summed, k);
            // entry e of lane j is pick E * j + e; only picks below `limit` count
            bool hm[WALK_E];
#pragma unroll
            for (int e = 0; e < WALK_E; ++e) hm[e] = !(x[e] < target) && WALK_E * lane + e < limit;
            const int hit = walk_first(hm);
            const bool reached = hit < WALK_RUN;
            const int taken = reached ? hit + 1 : limit;                    // picks applied
            if (taken > 0) {
                const int te = (taken - 1) % WALK_E;
                float xs = x[0];
#pragma unroll
                for (int e = 1; e < WALK_E; ++e) xs = te == e ? x[e] : xs;
                sum = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, xs), (taken - 1) / WALK_E));
            }
            cnt_s += which == 0 ? taken : 0;
            cnt_v += which == 0 ? 0 : taken;
            if (!reached && last) { all = true; break; }  // the pick after the last one has no positive gain
        }
        if (lane == 0) {
            walk_st(&sync->stop, 1);
            if (failed) walk_st(&sync->err, 1);
            // A wait that ran into its bound (never observed with the default bound) reports the conservative
            // result, every line selected: the coverage target of Alg. 2 still holds for it, and the context's
            // status word tells the caller.
            a.s_cnt[bh] = (failed || all) ? n : cnt_s;
            a.v_cnt[bh] = (failed || all) ? n : cnt_v;
            if (failed) atomicOr(a.status, STAT_WALK_TIMEOUT);
            if (a.accounted) a.accounted[bh] = sum;
        }
        return;
    }

    // ---------------------------------------------------------------------- the decisions (wave 0)
    const bool early = a.accounted == nullptr;
    int is = 0, iv = 0;                        // heads of the two lists (plain scalars: an array indexed by the
    int blk_s = 0, blk_v = 0;                  // list would be kept in scratch memory); block each head is in
    int have_s = 0, have_v = 0;                // blocks of each list known to be resident (staged and summed)
    int published = 0;                         // runs handed to the summing wave
    bool failed = false;

    // until the head's block and the one after it (the first `want` blocks of list l) are resident
    auto wait_blocks = [&](int l, int want) {
        int spins = 0, have;
        for (;;) {
            const int st = walk_ld(&sync->staged[l]), su = walk_ld(&sync->summed_blk[l]);
            have = st < su ? st : su;
            if (have >= want) break;
            __builtin_amdgcn_s_sleep(1);
            if (++spins > spin_limit || walk_ld(&sync->err)) { failed = true; break; }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        return have;
    };

    // What the lanes need of a list when its head is at `h`: lane l looks at the entries h + E l .. h + E l + E - 1
    // (weight, overlap prefix, length), every lane at the head's own three values.  Re-read only when the head of
    // that list moves.  (All of them lie in the head's block or the one after it.)
    struct View { float cw[WALK_E], pre[WALK_E], cl[WALK_E], w0, l0, ol0; bool ok[WALK_E], has; };
    auto view = [&](int l, int h) {
        const WalkList& L = lists[l];
        View r;
#pragma unroll
        for (int e = 0; e < WALK_E; ++e) {
            const int i = h + WALK_E * lane + e;
            r.ok[e] = i < n;
            const int ii = (i < n ? i : n - 1) & (WALK_CAP - 1);           // nothing is read from a block that never comes
            r.cw[e] = L.cw[ii]; r.pre[e] = L.pre[ii]; r.cl[e] = L.cl[ii];
        }
        r.has = h < n;
        const int hh = (r.has ? h : n - 1) & (WALK_CAP - 1);
        r.w0 = r.has ? L.cw[hh] : 0.f;                     // an exhausted list: no weight, and its overlap sum
        r.l0 = r.has ? L.cl[hh] : 1.f;                     // sits right behind its last line
        r.ol0 = r.has ? L.pre[hh] : sync->tot[l];
        return r;
    };
    // blocks a view at head h reads: through the block of entry h + RUN - 1, and pre[h] itself
    auto blocks_for = [&](int h) {
        const int want = (h + WALK_RUN - 1) / WALK_BLK + 1;
        return want < nblk ? want : nblk;
    };
    have_s = wait_blocks(0, blocks_for(0));
    have_v = wait_blocks(1, blocks_for(0));
    View S = view(0, 0), V = view(1, 0);

    while (!failed) {
        if (is >= n && iv >= n) break;
        // a head that has entered a new block frees the blocks behind it; a view that reaches into a block not
        // known to be resident yet is read again once that block is
        if (is / WALK_BLK != blk_s && is < n) {
            blk_s = is / WALK_BLK;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");         // done reading the blocks left behind
            if (lane == 0) walk_st(&sync->cur[0], blk_s);
        }
        if (iv / WALK_BLK != blk_v && iv < n) {
            blk_v = iv / WALK_BLK;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            if (lane == 0) walk_st(&sync->cur[1], blk_v);
        }
        if (is < n && have_s < blocks_for(is)) {
            have_s = wait_blocks(0, blocks_for(is));
            if (failed) break;
            S = view(0, is);
        }
        if (iv < n && have_v < blocks_for(iv)) {
            have_v = wait_blocks(1, blocks_for(iv));
            if (failed) break;
            V = view(1, iv);
        }
        const bool s_has = S.has, v_has = V.has;
        // entry e of lane j: the decision if the walk has taken E j + e more slashes (iv frozen)
        float gain[WALK_E];
        bool turn[WALK_E], dead[WALK_E];           // the pick goes to the other list; no gain is left
#pragma unroll
        for (int e = 0; e < WALK_E; ++e) {
            const int i = is + WALK_E * lane + e;
            const float ds = __fsub_rn(S.cw[e], V.ol0);
            const float dv = __fsub_rn(V.w0, S.pre[e]);
            float cs = __fsub_rn(S.cl[e], (float)iv); if (cs < 1.0f) cs = 1.0f;
            float cv = __fsub_rn(V.l0, (float)i); if (cv < 1.0f) cv = 1.0f;
            turn[e] = !(S.ok[e] && (!v_has || __fmul_rn(ds, cv) >= __fmul_rn(dv, cs)));
            dead[e] = !(ds > 0.f) && (!v_has || !(dv > 0.f));
            gain[e] = ds;
        }
        int run = walk_first(turn);
        int which = 0;
        if (run == 0) {
            // the head pick is a vertical; entry e of lane j: the decision if E j + e more verticals are taken (is frozen)
            which = 1;
#pragma unroll
            for (int e = 0; e < WALK_E; ++e) {
                const int i = iv + WALK_E * lane + e;
                const float dv = __fsub_rn(V.cw[e], S.ol0);
                const float ds = __fsub_rn(S.w0, V.pre[e]);
                float cv = __fsub_rn(V.cl[e], (float)is); if (cv < 1.0f) cv = 1.0f;
                float cs = __fsub_rn(S.l0, (float)i); if (cs < 1.0f) cs = 1.0f;
                turn[e] = !(V.ok[e] && !(s_has && __fmul_rn(ds, cv) >= __fmul_rn(dv, cs)));           // true: not a vertical again
                dead[e] = !(dv > 0.f) && (!s_has || !(ds > 0.f));
                gain[e] = dv;
            }
            run = walk_first(turn);
        }
        if (run == 0) break;                   // cannot happen (entry 0 of lane 0 repeats the head's test); never spin
        // picks 0 .. run-1 come from list `which`; the walk ends early at a pick with no positive gain left
        int stop_dead = WALK_RUN;
        if (early) stop_dead = walk_first(dead);
        const int limit = run < stop_dead ? run : stop_dead;
        // the list's view after the run (read again above if it reaches into a block that is not resident yet)
        const View nxt = view(which, (which == 0 ? is : iv) + limit);
        // hand the run over: a free slot of the ring, the gains, then the count of published runs
        bool stopped = false;
        int spins = 0;
        for (;;) {                             // one read: runs taken out of the ring, and whether the walk is over
            const unsigned long long ss = __atomic_load_n(static_cast<const unsigned long long*>(__builtin_assume_aligned(&sync->summed, 8)), __ATOMIC_RELAXED);
            if (__builtin_amdgcn_readfirstlane((int)(ss >> 32))) { stopped = true; break; }
            if (published - __builtin_amdgcn_readfirstlane((int)ss) < WALK_RING) break;
            __builtin_amdgcn_s_sleep(1);
            if (++spins > spin_limit || walk_ld(&sync->err)) { failed = true; break; }
        }
        if (stopped || failed) break;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        WalkRun& R = ring[published & (WALK_RING - 1)];
#pragma unroll
        for (int e = 0; e < WALK_E; e += 2)
            *reinterpret_cast<float2*>(&R.g[WALK_E * lane + e]) = make_float2(gain[e], gain[e + 1]);
        if (lane == 0) { R.which = which; R.limit = limit; R.last = stop_dead < run ? 1 : 0; }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        ++published;
        if (lane == 0) walk_st(&sync->runs, published);
        if (stop_dead < run) break;            // nothing after this run can add to the sum
        if (which == 0) { is += limit; S = nxt; } else { iv += limit; V = nxt; }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    if (lane == 0) {
        if (failed) walk_st(&sync->err, 1);
        walk_st(&sync->decided, 1);
        walk_st(&sync->done, 1);
    }
}

// ---- Alg. 2 with the overlap of a candidate counted cell by cell ----------------------------------
// The loop of Alg. 2 compares the marginal contributions of the two list heads (Sec. 5.1); the listing bounds the
// part of a line that is already covered by the sum of w^max of the lines taken from the other list.  This variant
// adds that part up exactly: a diagonal o and a column b share the cell of the scored row at position b + o, if
// there is one, so
//     overlap(slash o)  = sum over scored rows t with key c = p_t - o >= 0 and c taken  of A[t][c]
//     overlap(column b) = sum over scored rows t with o = p_t - b >= 0 and o taken      of A[t][b]
// "Taken" is a comparison of ranks: the lists are used up from the front, so column c is taken iff its position
// in the sorted column list is below the number of columns taken so far.  A candidate therefore needs, once, the
// w cells of its line and the ranks of the w lines it crosses; its overlap at any later moment is a masked sum of
// those cells.  Everything else is the loop of walk_kernel (binary32, single roundings, cross-multiplied test).
//
// rank_kernel: inverse of the sorted order, rank[list][bh][line] = position of the line in its sorted list.
__global__ void rank_kernel(SelectArgs a) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t seg = ((int64_t)blockIdx.z * a.BH + blockIdx.y) * a.n;
    if (i < a.n) a.sidx0[seg + a.sidx1[seg + i]] = (int32_t)i;
}

constexpr int XW_STAGERS = 3;                  // staging waves per list
constexpr int XW_THREADS = 64 * (1 + 2 * XW_STAGERS);   // wave 0 walks, then XW_STAGERS waves per list stage its records
constexpr int XW_CELLS = 4096;                 // cells of staged records per list: a ring of XW_CELLS / wpad records
constexpr int XW_BATCH = 8;                    // records a stager fetches per round trip
struct XwSync { int staged[2], head[2], done, err; };

// Sum of a double over the 64 lanes, the same value in every lane.  Data-parallel-primitive moves on the two
// halves of the value instead of cross-lane reads through LDS: a shuffle of a double is two LDS round trips, six
// steps of them were most of the time of a pick.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_f64(double x) {      // lanes outside ROW_MASK receive 0
    const uint64_t u = __builtin_bit_cast(uint64_t, x);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)u, CTRL, ROW_MASK, 0xF, false);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(u >> 32), CTRL, ROW_MASK, 0xF, false);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ double wave_sum_f64(double x) {
    x += dpp_f64<0xB1, 0xF>(x);                            // quad_perm [1,0,3,2]
    x += dpp_f64<0x4E, 0xF>(x);                            // quad_perm [2,3,0,1]: every lane holds its quad's sum
    x += dpp_f64<0x141, 0xF>(x);                           // row_half_mirror: sums of 8
    x += dpp_f64<0x140, 0xF>(x);                           // row_mirror: every lane holds its row's (16 lanes) sum
    x += dpp_f64<0x142, 0xA>(x);                           // row_bcast15 into rows 1 and 3
    x += dpp_f64<0x143, 0xC>(x);                           // row_bcast31 into rows 2 and 3: lane 63 holds the total
    const uint64_t u = __builtin_bit_cast(uint64_t, x);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)u, 63), hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(u >> 32), 63);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

// grid (BH).  LDS: per list a ring of records (wpad cells + wpad ranks each) and per-record line index / weight.
// NC: cells of a record per lane held in registers (1, 2 or 4; a window of w rows needs ceil(w / 64))
template <int NC>
__global__ __launch_bounds__(XW_THREADS) void walk_exact_kernel(SelectArgs a) {
    extern __shared__ __align__(16) unsigned char xw_lds[];
    const int W = a.w, wpad = (W + 63) / 64 * 64, CP = wpad / 64, ring = XW_CELLS / wpad;      // ring >= 16 (w <= 256)
    float* cells = reinterpret_cast<float*>(xw_lds);                       // [2][ring][wpad]
    int32_t* ranks = reinterpret_cast<int32_t*>(cells + 2 * XW_CELLS);     // [2][ring][wpad]
    int32_t* ridx = ranks + 2 * XW_CELLS;                                  // [2][ring] line index of a record
    float* rwt = reinterpret_cast<float*>(ridx + 2 * 256);                 // [2][ring] its weight
    XwSync* sync = reinterpret_cast<XwSync*>(rwt + 2 * 256);
    const int bh = blockIdx.x, lane = threadIdx.x & 63;
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = (int)a.n;
    const int spin_limit = a.spin_limit;
    if (threadIdx.x == 0) { sync->staged[0] = sync->staged[1] = 0; sync->head[0] = sync->head[1] = 0; sync->done = 0; sync->err = 0; }
    __syncthreads();

    if (wv != 0) {
        // ------------------------------------------------------------------ staging of one list
        // XW_STAGERS waves per list take the batches of XW_BATCH records in turn (stager s: batches s, s + S, ...),
        // so that the memory round trips of consecutive batches overlap; a batch is published in order, once the
        // batch before it has been.
        const int l = (wv - 1) / XW_STAGERS, sidx = (wv - 1) % XW_STAGERS; // list (0: slashes, 1: columns), stager
        const int32_t* sorted = a.sidx1 + ((int64_t)l * a.BH + bh) * a.n;
        const int32_t* rank_other = a.sidx0 + ((int64_t)(1 - l) * a.BH + bh) * a.n;
        const float* wts = (l == 0 ? a.slash : a.vert) + (int64_t)bh * a.n;
        const float* A = a.a_win + (int64_t)bh * W * a.n;
        int pos[NC];                                                        // positions of this lane's rows t = lane + 64 c
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const int t = lane + 64 * c;
            int64_t p = t < W ? (a.q_pos ? a.q_pos[t] : (int64_t)n - W + t) : -1;
            if (p > n - 1) p = n - 1;
            pos[c] = (int)p;
        }
        for (int j = sidx * XW_BATCH; j < n; j += XW_STAGERS * XW_BATCH) {
            const int batch = n - j < XW_BATCH ? n - j : XW_BATCH;
            // the loads do not depend on the ring: issued before waiting for room
            int32_t idx[XW_BATCH];
#pragma unroll
            for (int r = 0; r < XW_BATCH; ++r) idx[r] = sorted[j + (r < batch ? r : 0)];
            float wt[XW_BATCH], cell[XW_BATCH][NC];
            int32_t rk[XW_BATCH][NC];
#pragma unroll
            for (int r = 0; r < XW_BATCH; ++r) {
                wt[r] = wts[idx[r]];
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    cell[r][c] = 0.f; rk[r][c] = 0x7FFFFFFF;
                    if (c < CP) {
                        const int t = lane + 64 * c;
                        const int other = pos[c] - idx[r];                 // the crossed line of the other kind (key, or diagonal)
                        if (t < W && other >= 0) {
                            const int key = l == 0 ? other : idx[r];
                            cell[r][c] = A[(int64_t)t * a.n + key];
                            rk[r][c] = rank_other[other];
                        }
                    }
                }
            }
            // room for the whole batch: its last record may be written once record j + batch - 1 - ring has been left
            bool stop = false;
            for (int spins = 0; walk_ld(&sync->head[l]) + ring < j + batch; ) {
                if (walk_ld(&sync->done) != 0) { stop = true; break; }
                __builtin_amdgcn_s_sleep(2);
                if (++spins > spin_limit) { walk_st(&sync->err, 1); stop = true; break; }
            }
            if (stop) break;
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
#pragma unroll
            for (int r = 0; r < XW_BATCH; ++r) {
                if (r < batch) {
                    const int slot = (j + r) % ring;
#pragma unroll
                    for (int c = 0; c < NC; ++c)
                        if (c < CP) {
                            cells[(l * ring + slot) * wpad + lane + 64 * c] = cell[r][c];
                            ranks[(l * ring + slot) * wpad + lane + 64 * c] = rk[r][c];
                        }
                    if (lane == 0) { ridx[l * 256 + slot] = idx[r]; rwt[l * 256 + slot] = wt[r]; }
                }
            }
            // in-order publication: wait until every earlier batch is out
            for (int spins = 0; walk_ld(&sync->staged[l]) != j; ) {
                if (walk_ld(&sync->done) != 0) { stop = true; break; }
                __builtin_amdgcn_s_sleep(1);
                if (++spins > spin_limit) { walk_st(&sync->err, 1); stop = true; break; }
            }
            if (stop) break;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __builtin_amdgcn_wave_barrier();
            if (lane == 0) walk_st(&sync->staged[l], j + batch);
        }
        return;
    }

    // ---------------------------------------------------------------------- the walk (wave 0)
    const float target = a.alpha * a.total[bh];
    const float nh = (float)a.n_hat;
    float sum = 0.f;
    int is = 0, iv = 0;
    bool failed = false;
    // head record of each list, read again only when that head moves
    float c_s[NC], c_v[NC], w_s = 0.f, w_v = 0.f, l_s = 1.f, l_v = 1.f;
    int32_t r_s[NC], r_v[NC];
    int seen[2] = {0, 0};                                  // records of each list known to be staged (the counter is re-read only past that)
    auto wait_record = [&](int l, int want) {              // until record `want` of list l is staged
        if (want < seen[l]) return;
        int spins = 0, st;
        while ((st = walk_ld(&sync->staged[l])) <= want) {
            __builtin_amdgcn_s_sleep(1);
            if (++spins > spin_limit || walk_ld(&sync->err)) { failed = true; break; }
        }
        seen[l] = st;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    };
    auto read_record = [&](int l, int h, float (&c)[NC], int32_t (&r)[NC], float& wt, float& len) {
        const int slot = h % ring;
#pragma unroll
        for (int q = 0; q < NC; ++q) {
            c[q] = 0.f; r[q] = 0x7FFFFFFF;
            if (q < CP) { c[q] = cells[(l * ring + slot) * wpad + lane + 64 * q]; r[q] = ranks[(l * ring + slot) * wpad + lane + 64 * q]; }
        }
        const int line = ridx[l * 256 + slot];
        wt = rwt[l * 256 + slot];
        const float rest = (float)(n - line);
        len = rest < nh ? rest : nh;
    };
    auto overlap = [&](const float (&c)[NC], const int32_t (&r)[NC], int taken_other) -> float {
        double x = 0.0;
        bool any = false;
#pragma unroll
        for (int q = 0; q < NC; ++q) { const bool in = r[q] < taken_other; any |= in; x += in ? (double)c[q] : 0.0; }
        if (__ballot(any) == 0ull) return 0.f;             // no crossed line taken yet: nothing to add up
        return (float)wave_sum_f64(x);
    };
    // the heads are published (slots handed back to the stagers) every eighth pick
    if (n > 0) { wait_record(0, 0); wait_record(1, 0); }
    if (!failed) { read_record(0, 0, c_s, r_s, w_s, l_s); read_record(1, 0, c_v, r_v, w_v, l_v); }
    float ol_s = 0.f, ol_v = 0.f;
    bool dirty_s = true, dirty_v = true;
    auto crosses = [&](const int32_t (&r)[NC], int rank) -> bool {       // does the line of that rank cross this head's cells?
        bool hit = false;
#pragma unroll
        for (int q = 0; q < NC; ++q) hit |= r[q] == rank;
        return __ballot(hit) != 0ull;
    };
    int picks = 0;
    while (!failed && sum < target && (is < n || iv < n)) {
        const bool has_s = is < n, has_v = iv < n;
        // an overlap is summed again only when its set of taken crossed lines changed: a new list head, or the
        // line just taken from the other list crosses this head inside the window
        if (has_s && dirty_s) { ol_s = overlap(c_s, r_s, iv); dirty_s = false; }
        if (has_v && dirty_v) { ol_v = overlap(c_v, r_v, is); dirty_v = false; }
        const float ds = has_s ? __fsub_rn(w_s, ol_s) : 0.f;
        const float dv = has_v ? __fsub_rn(w_v, ol_v) : 0.f;
        bool take_s;
        if (!has_v) take_s = true;
        else if (!has_s) take_s = false;
        else {
            float cs = __fsub_rn(l_s, (float)iv); if (cs < 1.0f) cs = 1.0f;
            float cv = __fsub_rn(l_v, (float)is); if (cv < 1.0f) cv = 1.0f;
            take_s = __fmul_rn(ds, cv) >= __fmul_rn(dv, cs);
        }
        if (take_s) {
            sum = __fadd_rn(sum, ds);
            ++is;
            dirty_s = true;
            dirty_v = dirty_v || crosses(r_v, is - 1);
            if (is < n && !(sum >= target)) { wait_record(0, is); if (!failed) read_record(0, is, c_s, r_s, w_s, l_s); }
        } else {
            sum = __fadd_rn(sum, dv);
            ++iv;
            dirty_v = true;
            dirty_s = dirty_s || crosses(r_s, iv - 1);
            if (iv < n && !(sum >= target)) { wait_record(1, iv); if (!failed) read_record(1, iv, c_v, r_v, w_v, l_v); }
        }
        if ((++picks & 7) == 0) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");         // done reading the records left behind
            if (lane == 0) { walk_st(&sync->head[0], is); walk_st(&sync->head[1], iv); }
        }
    }
    if (lane == 0) {
        if (failed) { walk_st(&sync->err, 1); atomicOr(a.status, STAT_WALK_TIMEOUT); }
        walk_st(&sync->done, 1);
        // a wait that ran into its bound reports every line selected (the coverage target still holds)
        a.s_cnt[bh] = failed ? n : is;
        a.v_cnt[bh] = failed ? n : iv;
        if (a.accounted) a.accounted[bh] = sum;
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
    if (tid == 0 && cnt > cap) atomicOr(a.status, list == 0 ? STAT_S_TRUNCATED : STAT_V_TRUNCATED);
    if (cnt >= n) {                                        // every line was taken: the list is 0 .. n-1
        for (int64_t i = tid; i < n && i < cap; i += 1024) out[i] = (int32_t)i;
        return;
    }
    for (int i = tid; i < words; i += 1024) bm[i] = 0u;
    if (tid == 0) carry = 0u;
    __syncthreads();
    for (int i0 = tid; i0 < cnt; i0 += 8 * 1024) {          // eight independent loads in flight per thread
        int32_t x8[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) { const int i = i0 + j * 1024; x8[j] = i < cnt ? sorted_idx[i] : -1; }
#pragma unroll
        for (int j = 0; j < 8; ++j) if (x8[j] >= 0) atomicOr(&bm[x8[j] >> 5], 1u << (x8[j] & 31));
    }
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

// ---- union of two selections ------------------------------------------------------------------------
// Alg. 1 keeps the lines selected in every turn so far (its set L); Sec. 5, Step 1 notes that selected lines can be
// reused in later turns.  Column indices are key positions and diagonal indices are offsets, both unchanged when the
// context grows, so carrying a selection into a later turn is a union of index sets.  grid (2, BH): list 0 =
// diagonals, list 1 = columns; both inputs are marked in an LDS bitmap of n bits, which is then written out in order.
__global__ __launch_bounds__(1024) void merge_lines_kernel(MergeArgs a) {
    extern __shared__ uint32_t bm[];
    __shared__ uint32_t wsum[16];
    __shared__ uint32_t carry;
    const int list = blockIdx.x, bh = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int64_t n = a.n;
    const int words = (int)((n + 31) / 32);
    for (int i = tid; i < words; i += 1024) bm[i] = 0u;
    if (tid == 0) carry = 0u;
    __syncthreads();
    bool dropped = false;
    for (int src = 0; src < 2; ++src) {
        const int32_t* idx = (src ? a.idx_b[list] : a.idx_a[list]) + (int64_t)bh * (src ? a.cap_b[list] : a.cap_a[list]);
        int cnt = (src ? a.cnt_b[list] : a.cnt_a[list])[bh];
        const int cap = src ? a.cap_b[list] : a.cap_a[list];
        if (cnt > cap) cnt = cap;
        for (int i = tid; i < cnt; i += 1024) {
            const int32_t x = idx[i];
            if (x >= 0 && x < n) atomicOr(&bm[x >> 5], 1u << (x & 31)); else dropped = true;
        }
    }
    dropped = __syncthreads_or(dropped);
    int32_t* out = a.idx[list] + (int64_t)bh * a.cap[list];
    const int cap = a.cap[list];
    uint32_t total = 0;
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
        if (tid == 1023) { carry = pre + inc; }
        __syncthreads();
        total = carry;
    }
    if (tid == 0) {
        a.cnt[list][bh] = (int32_t)total;
        if (total > (uint32_t)cap) atomicOr(a.status, list == 0 ? STAT_S_TRUNCATED : STAT_V_TRUNCATED);
        if (dropped) atomicOr(a.status, STAT_MERGE_RANGE);
    }
}

hipError_t run_merge_lines(const MergeArgs& a, hipStream_t st) {
    const size_t smem = (size_t)((a.n + 31) / 32) * 4;
    hipLaunchKernelGGL(merge_lines_kernel, dim3(2, a.BH), dim3(1024), smem, st, a);
    return hipGetLastError();
}

// ---- top-B retention ------------------------------------------------------------------------------
// keep_idx [BK][budget] ascending; keep_cnt = min(budget, len).
// Radix select on the descending keys in three digits (11 + 11 + 10 bits, most significant first) finds the
// key K* of the budget-th largest score; then every element above K* and the first few equal to it are
// written in index order.  One KV head has too few elements to need a chip but too many for one CU to be
// quick, so a head's scores are cut into chunks of TB_CHUNK, one workgroup each, and the steps are separate
// launches that meet in small global arrays: hist [BK][3][TB_BINS] (zeroed by the first launch), state
// [BK][3][2] (prefix and elements still wanted after each digit) and cnt [BK][chunks][2].
constexpr int TB_THREADS = 1024;
constexpr int TB_CHUNK = 2048;
constexpr int TB_BINS = 2048;

__device__ __forceinline__ uint32_t tb_digit(uint32_t key, int pass) {
    return pass == 0 ? key >> 21 : pass == 1 ? (key >> 10) & 2047u : key & 1023u;
}
__device__ __forceinline__ uint32_t tb_himask(int pass) { return pass == 0 ? 0u : pass == 1 ? 0xFFE00000u : 0xFFFFFC00u; }
__device__ __forceinline__ int tb_shift(int pass) { return pass == 0 ? 21 : pass == 1 ? 10 : 0; }

// All threads of a workgroup: from the histogram of digit `pass` (among the keys that match `prefix`) and the
// number of elements still wanted, the digit that holds the wanted-th element; returns the longer prefix and
// what is still wanted inside it.
__device__ __forceinline__ void tb_pick(const uint32_t* hist, int pass, uint32_t prefix, uint32_t rem,
                                        uint32_t* wsum, uint32_t* res, uint32_t& prefix_out, uint32_t& rem_out) {
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const uint32_t h0 = hist[2 * tid], h1 = hist[2 * tid + 1];
    const uint32_t v = h0 + h1;
    uint32_t inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) { const uint32_t t = __shfl_up(inc, off, 64); if (lane >= off) inc += t; }
    __syncthreads();                                       // wsum / res may still be read from an earlier call
    if (lane == 63) wsum[wv] = inc;
    __syncthreads();
    uint32_t ex = inc - v;
    for (int w = 0; w < wv; ++w) ex += wsum[w];
    if (ex < rem && rem <= ex + v) {                       // exactly one thread: the total is at least rem
        const uint32_t r = rem - ex;
        const uint32_t d = 2u * tid + (r > h0 ? 1u : 0u);
        res[0] = prefix | (d << tb_shift(pass));
        res[1] = r > h0 ? r - h0 : r;
    }
    __syncthreads();
    prefix_out = res[0]; rem_out = res[1];
}

__global__ void topb_zero_kernel(uint32_t* p, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0u;
}

// grid (chunks, BK): histogram of digit PASS over this chunk's keys that match the prefix found so far
template <int PASS>
__global__ __launch_bounds__(TB_THREADS) void topb_hist_kernel(TopbArgs a) {
    __shared__ uint32_t lh[TB_BINS];
    __shared__ uint32_t wsum[16], res[2];
    const int chunk = blockIdx.x, bk = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
    const int64_t len = a.len;
    const int64_t keep = a.budget < len ? a.budget : len;
    if (keep == len) return;                               // everything is kept: the write step needs no threshold
    uint32_t* hist = a.hist + (int64_t)bk * 3 * TB_BINS;
    uint32_t* state = a.state + (int64_t)bk * 6;
    uint32_t prefix = 0u, rem = (uint32_t)keep;
    if (PASS >= 1) {
        if (PASS == 2) { prefix = state[0]; rem = state[1]; }
        tb_pick(hist + (PASS - 1) * TB_BINS, PASS - 1, prefix, rem, wsum, res, prefix, rem);
        if (chunk == 0 && tid == 0) { state[2 * (PASS - 1)] = prefix; state[2 * (PASS - 1) + 1] = rem; }
    }
    for (int i = tid; i < TB_BINS; i += TB_THREADS) lh[i] = 0u;
    __syncthreads();
    const float* sc = a.score + (int64_t)bk * len;
    uint32_t kb[TB_CHUNK / TB_THREADS];
#pragma unroll
    for (int q = 0; q < TB_CHUNK / TB_THREADS; ++q) {
        const int64_t i = (int64_t)chunk * TB_CHUNK + q * TB_THREADS + tid;
        kb[q] = i < len ? desc_key(sc[i]) : 0xFFFFFFFFu;
    }
#pragma unroll
    for (int q = 0; q < TB_CHUNK / TB_THREADS; ++q) {
        // scores of one head crowd into few digits: lanes with the same digit add once, through their first lane
        const int64_t i = (int64_t)chunk * TB_CHUNK + q * TB_THREADS + tid;
        const bool on = i < len && (kb[q] & tb_himask(PASS)) == prefix;
        const uint32_t digit = tb_digit(kb[q], PASS);
        uint64_t peers = __ballot(on);
#pragma unroll
        for (int b = 0; b < 11; ++b) {
            const bool bit = (digit >> b) & 1u;
            const uint64_t m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        if (on && __ffsll((unsigned long long)peers) - 1 == lane) atomicAdd(&lh[digit], (uint32_t)__popcll(peers));
    }
    __syncthreads();
    for (int i = tid; i < TB_BINS; i += TB_THREADS) if (lh[i]) atomicAdd(&hist[PASS * TB_BINS + i], lh[i]);
}

// grid (chunks, BK): K* and the number of elements equal to it that are kept; per chunk, how many of its
// elements lie above K* and how many equal it
__global__ __launch_bounds__(TB_THREADS) void topb_count_kernel(TopbArgs a) {
    __shared__ uint32_t wsum[16], res[2], wg[16], we[16];
    const int chunk = blockIdx.x, bk = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int64_t len = a.len;
    const int64_t keep = a.budget < len ? a.budget : len;
    if (keep == len) return;
    uint32_t* state = a.state + (int64_t)bk * 6;
    uint32_t kstar, need_eq;
    tb_pick(a.hist + ((int64_t)bk * 3 + 2) * TB_BINS, 2, state[2], state[3], wsum, res, kstar, need_eq);
    if (chunk == 0 && tid == 0) { state[4] = kstar; state[5] = need_eq; }
    const float* sc = a.score + (int64_t)bk * len;
    uint32_t g = 0, e = 0;
#pragma unroll
    for (int q = 0; q < TB_CHUNK / TB_THREADS; ++q) {
        const int64_t i = (int64_t)chunk * TB_CHUNK + q * TB_THREADS + tid;
        const uint32_t key = i < len ? desc_key(sc[i]) : 0xFFFFFFFFu;
        g += (uint32_t)__popcll(__ballot(i < len && key < kstar));
        e += (uint32_t)__popcll(__ballot(i < len && key == kstar));
    }
    if (lane == 0) { wg[wv] = g; we[wv] = e; }
    __syncthreads();
    if (tid == 0) {
        uint32_t tg = 0, te = 0;
        for (int w = 0; w < 16; ++w) { tg += wg[w]; te += we[w]; }
        a.cnt[((int64_t)bk * a.chunks + chunk) * 2] = tg;
        a.cnt[((int64_t)bk * a.chunks + chunk) * 2 + 1] = te;
    }
}

// grid (chunks, BK): slot of a kept element = kept elements before it; kept = above K*, or equal to it among
// the first need_eq of those
__global__ __launch_bounds__(TB_THREADS) void topb_write_kernel(TopbArgs a) {
    __shared__ uint32_t seg_g[TB_CHUNK / 64], seg_e[TB_CHUNK / 64], base_s[2];
    const int chunk = blockIdx.x, bk = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int64_t len = a.len;
    const int64_t keep = a.budget < len ? a.budget : len;
    int32_t* out = a.keep_idx + (int64_t)bk * a.budget;
    if (chunk == 0 && tid == 0) a.keep_cnt[bk] = (int32_t)keep;
    if (keep == len) {
#pragma unroll
        for (int q = 0; q < TB_CHUNK / TB_THREADS; ++q) {
            const int64_t i = (int64_t)chunk * TB_CHUNK + q * TB_THREADS + tid;
            if (i < len) out[i] = (int32_t)i;
        }
        return;
    }
    const uint32_t* state = a.state + (int64_t)bk * 6;
    const uint32_t kstar = state[4], need_eq = state[5];
    const float* sc = a.score + (int64_t)bk * len;
    // elements above / equal to K* in the chunks before this one (one wave adds them up, lanes striding)
    if (wv == 0) {
        uint32_t g = 0, e = 0;
        for (int c = lane; c < chunk; c += 64) { g += a.cnt[((int64_t)bk * a.chunks + c) * 2]; e += a.cnt[((int64_t)bk * a.chunks + c) * 2 + 1]; }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) { g += __shfl_xor(g, off, 64); e += __shfl_xor(e, off, 64); }
        if (lane == 0) { base_s[0] = g; base_s[1] = e; }
    }
    uint32_t kb[TB_CHUNK / TB_THREADS];
#pragma unroll
    for (int q = 0; q < TB_CHUNK / TB_THREADS; ++q) {
        const int64_t i = (int64_t)chunk * TB_CHUNK + q * TB_THREADS + tid;
        kb[q] = i < len ? desc_key(sc[i]) : 0xFFFFFFFFu;
        const uint64_t gm = __ballot(i < len && kb[q] < kstar), em = __ballot(i < len && kb[q] == kstar);
        if (lane == 0) { seg_g[q * 16 + wv] = (uint32_t)__popcll(gm); seg_e[q * 16 + wv] = (uint32_t)__popcll(em); }
    }
    __syncthreads();
    if (wv == 0) {                                         // exclusive scan over the chunk's 64-element segments
        uint32_t g = lane < TB_CHUNK / 64 ? seg_g[lane] : 0u, e = lane < TB_CHUNK / 64 ? seg_e[lane] : 0u;
        uint32_t ig = g, ie = e;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t ug = __shfl_up(ig, off, 64), ue = __shfl_up(ie, off, 64);
            if (lane >= off) { ig += ug; ie += ue; }
        }
        if (lane < TB_CHUNK / 64) { seg_g[lane] = base_s[0] + ig - g; seg_e[lane] = base_s[1] + ie - e; }
    }
    __syncthreads();
    const uint64_t below = (1ull << lane) - 1ull;
#pragma unroll
    for (int q = 0; q < TB_CHUNK / TB_THREADS; ++q) {
        const int64_t i = (int64_t)chunk * TB_CHUNK + q * TB_THREADS + tid;
        const bool gt = i < len && kb[q] < kstar, eq = i < len && kb[q] == kstar;
        const uint64_t gm = __ballot(gt), em = __ballot(eq);
        const uint32_t gt_before = seg_g[q * 16 + wv] + (uint32_t)__popcll(gm & below);
        const uint32_t eq_before = seg_e[q * 16 + wv] + (uint32_t)__popcll(em & below);
        const uint32_t eq_kept_before = eq_before < need_eq ? eq_before : need_eq;
        if (gt || (eq && eq_before < need_eq)) out[gt_before + eq_kept_before] = (int32_t)i;
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

template <int SEG>
static hipError_t launch_sort(const SelectArgs& a, hipStream_t st) {
    const int nseg = (int)((a.n + SEG - 1) / SEG);
    hipLaunchKernelGGL(sort_seg_kernel<SEG>, dim3(nseg, 2, a.BH), dim3(SORT_THREADS), sort_lds_bytes(SEG), st, a);
    hipLaunchKernelGGL(sort_merge_kernel<SEG>, dim3(nseg, 2, a.BH), dim3(SORT_THREADS), 2 * SEG * 4, st, a);
    return hipGetLastError();
}

hipError_t init_select_kernels() {
    hipError_t e;
    if ((e = allow_full_lds(&sort_seg_kernel<SORT_SEG_MIN>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&sort_seg_kernel<4096>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&sort_seg_kernel<SORT_SEG_MAX>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&sort_merge_kernel<SORT_SEG_MIN>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&sort_merge_kernel<4096>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&sort_merge_kernel<SORT_SEG_MAX>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&walk_kernel)) != hipSuccess) return e;
    if ((e = allow_full_lds(&walk_exact_kernel<1>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&walk_exact_kernel<2>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&walk_exact_kernel<4>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&merge_lines_kernel)) != hipSuccess) return e;
    return allow_full_lds(&emit_kernel);
}

hipError_t run_select(const SelectArgs& a, hipStream_t st) {
    // Segment length: the merge's work per workgroup hardly depends on it, the sort's shrinks with it, so the
    // shortest one that still gives no more workgroups than the chip has compute units (256).
    const int64_t want = a.n * 2 * a.BH / 256;
    hipError_t e = want <= SORT_SEG_MIN ? launch_sort<SORT_SEG_MIN>(a, st)
                 : want <= 4096         ? launch_sort<4096>(a, st)
                                        : launch_sort<SORT_SEG_MAX>(a, st);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(walk_kernel, dim3(a.BH), dim3(WALK_THREADS), WALK_LDS_BYTES, st, a);
    const size_t smem = (size_t)((a.n + 31) / 32) * 4;
    hipLaunchKernelGGL(emit_kernel, dim3(2, a.BH), dim3(1024), smem, st, a);
    return hipGetLastError();
}

hipError_t run_select_exact(const SelectArgs& a, hipStream_t st) {
    const int64_t want = a.n * 2 * a.BH / 256;
    hipError_t e = want <= SORT_SEG_MIN ? launch_sort<SORT_SEG_MIN>(a, st)
                 : want <= 4096         ? launch_sort<4096>(a, st)
                                        : launch_sort<SORT_SEG_MAX>(a, st);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(rank_kernel, dim3((unsigned)((a.n + 255) / 256), a.BH, 2), dim3(256), 0, st, a);
    const size_t xw = 2 * XW_CELLS * 8 + 2 * 256 * 8 + sizeof(XwSync) + 16;
    if (a.w <= 64) hipLaunchKernelGGL(walk_exact_kernel<1>, dim3(a.BH), dim3(XW_THREADS), xw, st, a);
    else if (a.w <= 128) hipLaunchKernelGGL(walk_exact_kernel<2>, dim3(a.BH), dim3(XW_THREADS), xw, st, a);
    else hipLaunchKernelGGL(walk_exact_kernel<4>, dim3(a.BH), dim3(XW_THREADS), xw, st, a);
    const size_t smem = (size_t)((a.n + 31) / 32) * 4;
    hipLaunchKernelGGL(emit_kernel, dim3(2, a.BH), dim3(1024), smem, st, a);
    return hipGetLastError();
}

int topb_chunks(int64_t len) { return (int)((len + TB_CHUNK - 1) / TB_CHUNK); }
size_t topb_scratch_words(int BK, int64_t len) { return (size_t)BK * (3 * TB_BINS + 6 + 2 * (size_t)topb_chunks(len)); }

hipError_t run_topb(const TopbArgs& a0, int BK, uint32_t* scratch, hipStream_t st) {
    if (a0.len < 1 || a0.len > TOPB_MAX_LEN || a0.budget < 1) return hipErrorInvalidValue;
    TopbArgs a = a0;
    a.chunks = topb_chunks(a.len);
    a.hist = scratch;
    a.state = a.hist + (size_t)BK * 3 * TB_BINS;
    a.cnt = a.state + (size_t)BK * 6;
    const dim3 grid(a.chunks, BK);
    const int nz = BK * 3 * TB_BINS;
    hipLaunchKernelGGL(topb_zero_kernel, dim3((nz + 255) / 256), dim3(256), 0, st, a.hist, nz);
    hipLaunchKernelGGL(topb_hist_kernel<0>, grid, dim3(TB_THREADS), 0, st, a);
    hipLaunchKernelGGL(topb_hist_kernel<1>, grid, dim3(TB_THREADS), 0, st, a);
    hipLaunchKernelGGL(topb_hist_kernel<2>, grid, dim3(TB_THREADS), 0, st, a);
    hipLaunchKernelGGL(topb_count_kernel, grid, dim3(TB_THREADS), 0, st, a);
    hipLaunchKernelGGL(topb_write_kernel, grid, dim3(TB_THREADS), 0, st, a);
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
