// Window scoring: attention of the newest query window over the whole context, reduced to
// per-column ("vertical") and per-diagonal ("slash") sums and maxima (Alg. 2: the softmax step,
// SlashSum and VerticalSum; Sec. 3.1 defines the two kinds of line).  The same kernels, in
// "column sums only, summed over the query heads of a KV head" mode, produce the retention score
// of Alg. 3 (Sec. 5.2).
//
// The softmax normaliser of a row is only known after all keys were seen, and the line sums mix
// rows with different normalisers, so the pass is split:
//   stats_kernel   per (row, 128-key block): max and sum of exp of the scaled logits;
//   merge_kernel   per row: global max m and 1/l;
//   lines_kernel   recomputes the logits, forms A = exp2(x - m) / l, and reduces it
//                  - over rows, in registers, to column sums / maxima (written once, in order);
//                  - over diagonals through an LDS copy of the 128-key slab of A, one thread per
//                    diagonal adding the rows in fixed order; a diagonal crosses at most two key
//                    blocks, whose two partial results finish_kernel adds.
// Everything is summed in a fixed order, so results are bit-reproducible from run to run.
// With explicit scoring positions (q_pos given) the diagonals of a slab are not a contiguous
// range; that path uses fp32 atomics on zero-initialised outputs instead.
//
// Tile products run on 32x32 MFMA with K fragments held in registers (each wave owns 32 keys of
// the block and re-uses them for every query head of the KV group and every 32-row group).
#include "ls_device.h"
#include "ls_internal.h"

namespace ls {

constexpr int SB = 128;           // keys per workgroup
constexpr int SCORE_THREADS = 256;

template <typename T, int D>
__device__ __forceinline__ void load_k_frags(Frag<T> (&kf)[D / 16], const T* Kg, int64_t key, int64_t n, int g) {
    if (key < n) {
#pragma unroll
        for (int c = 0; c < D / 16; ++c) load_frag(kf[c], Kg + key * D + 16 * c + 8 * g);
    } else {
#pragma unroll
        for (int c = 0; c < D / 16; ++c) zero_frag(kf[c]);
    }
}

template <typename T, int D>
__device__ __forceinline__ void load_q_frags(Frag<T> (&qf)[D / 16], const T* Qh, int row, int w, int g) {
    if (row < w) {
#pragma unroll
        for (int c = 0; c < D / 16; ++c) load_frag(qf[c], Qh + (int64_t)row * D + 16 * c + 8 * g);
    } else {
#pragma unroll
        for (int c = 0; c < D / 16; ++c) zero_frag(qf[c]);
    }
}

// ---- the window's queries of one head, staged in LDS ---------------------------------------------
// Every workgroup of a KV head needs the same few KB of Q for each of its G heads; read straight from
// global memory by each wave (as the K fragments are) those reads all hit the same handful of L2 lines and
// took half of both passes.  One copy per workgroup and head goes through LDS instead: row-major, the
// 8-element fragment units of a row XOR-swizzled with the row so that the 16 rows one fragment read touches
// fall into different banks.  The next head's units are fetched into registers while the current head is
// multiplied.
template <typename T, int D>
struct QStage {
    static constexpr int FB = 8 * Elem<T>::bytes;         // bytes of one fragment unit (8 elements)
    static constexpr int UPR = D / 8;                     // units per row
    static constexpr int RBYTES = D * Elem<T>::bytes;
    static constexpr int PF = 4;                          // units per thread held in registers
    struct Unit { f32x4 v[FB / 16]; };
    __device__ static void fetch(Unit (&u)[PF], const T* Qh, int w, int wpad, int tid) {
#pragma unroll
        for (int j = 0; j < PF; ++j) {
            const int i = tid + SCORE_THREADS * j, row = i / UPR, uu = i % UPR;
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int h = 0; h < FB / 16; ++h)
                u[j].v[h] = (i < wpad * UPR && row < w) ? reinterpret_cast<const f32x4*>(Qh + (int64_t)row * D + 8 * uu)[h] : z;
        }
    }
    __device__ static unsigned char* slot(unsigned char* qs, int row, int uu) {
        return qs + row * RBYTES + FB * (uu ^ (row & (UPR - 1)));
    }
    // registers -> LDS; rows beyond the register budget (long windows) are copied directly
    __device__ static void commit(unsigned char* qs, const Unit (&u)[PF], const T* Qh, int w, int wpad, int tid) {
#pragma unroll
        for (int j = 0; j < PF; ++j) {
            const int i = tid + SCORE_THREADS * j, row = i / UPR, uu = i % UPR;
            if (i < wpad * UPR) {
#pragma unroll
                for (int h = 0; h < FB / 16; ++h) reinterpret_cast<f32x4*>(slot(qs, row, uu))[h] = u[j].v[h];
            }
        }
        for (int i = tid + SCORE_THREADS * PF; i < wpad * UPR; i += SCORE_THREADS) {
            const int row = i / UPR, uu = i % UPR;
            const f32x4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int h = 0; h < FB / 16; ++h)
                reinterpret_cast<f32x4*>(slot(qs, row, uu))[h] = row < w ? reinterpret_cast<const f32x4*>(Qh + (int64_t)row * D + 8 * uu)[h] : z;
        }
    }
    __device__ static void frags(Frag<T> (&qf)[D / 16], const unsigned char* qs, int row, int g) {
#pragma unroll
        for (int c = 0; c < D / 16; ++c) load_frag(qf[c], qs + row * RBYTES + FB * ((2 * c + g) ^ (row & (UPR - 1))));
    }
};

// ---- pass 1: per (row, key block) max and sum of exp2 -----------------------------------------
// grid (nkb, B*Hkv), dynamic LDS: the staged Q of one head.  part[(bh*w + row)*nkb + kb] = {max, sum}.
template <typename T, int D>
__global__ __launch_bounds__(SCORE_THREADS, (Elem<T>::bytes == 2 ? 4 : 1)) void stats_kernel(ScoreArgs a) {
    using QS = QStage<T, D>;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* qs = smem;                              // [wpad][D] staged queries
    __shared__ float red[2][4][32][2];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, r32 = lane & 31, g = lane >> 5;
    const int kb = blockIdx.x, bk = blockIdx.y;
    const int b = bk / a.Hkv, kvh = bk % a.Hkv;
    const int64_t n = a.n;
    const T* Kg = reinterpret_cast<const T*>(a.k) + (int64_t)bk * n * D;
    const int64_t key0 = (int64_t)kb * SB + 32 * wv;
    const int wpad = ((a.w + 31) / 32) * 32;
    const int rgs = wpad / 32;
    const int bh0 = b * a.Hq + kvh * a.G;
    const T* Q0 = reinterpret_cast<const T*>(a.q) + (int64_t)bh0 * a.w * D;
    typename QS::Unit qu[QS::PF];
    QS::fetch(qu, Q0, a.w, wpad, tid);
    Frag<T> kf[D / 16];
    load_k_frags<T, D>(kf, Kg, key0 + r32, n, g);
    // every key of the block is visible to every row of a contiguous window: no masks (all but the last blocks)
    const bool open = a.q_pos == nullptr && (int64_t)kb * SB + SB - 1 <= n - a.w;
    int it = 0;
    for (int gq = 0; gq < a.G; ++gq) {
        const int bh = bh0 + gq;
        const T* Qh = Q0 + (int64_t)gq * a.w * D;
        lds_barrier();                                     // the previous head's fragments have been read
        QS::commit(qs, qu, Qh, a.w, wpad, tid);
        lds_barrier();
        if (gq + 1 < a.G) QS::fetch(qu, Qh + (int64_t)a.w * D, a.w, wpad, tid);
        for (int rg = 0; rg < rgs; ++rg, ++it) {
            const int row = 32 * rg + r32;
            Frag<T> qf[D / 16];
            QS::frags(qf, qs, row, g);
            f32x16 s;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
            for (int c = 0; c < D / 16; ++c) mma(s, kf[c], qf[c]);   // s[r] = <k_{8(r/4)+4g+r%4}, q_row>
            float mx = -INFINITY;
            if (open && row < a.w) {
#pragma unroll
                for (int r = 0; r < 16; ++r) { s[r] *= a.scale_log2e; mx = fmaxf(mx, s[r]); }
            } else {
                int64_t p = (row < a.w) ? (a.q_pos ? a.q_pos[row] : n - a.w + row) : -1;
                if (p > n - 1) p = n - 1;                  // positions outside the context are clipped
                int64_t lim64 = p - key0 - 4 * g;          // register r holds key key0 + 4g + 8(r/4) + r%4
                const int lim = lim64 < -1 ? -1 : (lim64 > 64 ? 64 : (int)lim64);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float x = (8 * (r >> 2) + (r & 3) <= lim) ? s[r] * a.scale_log2e : -INFINITY;
                    s[r] = x;
                    mx = fmaxf(mx, x);
                }
            }
            mx = fmaxf(mx, xor32(mx));
            const float ms = (mx == -INFINITY) ? 0.f : mx;
            float sum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) sum += fast_exp2(s[r] - ms);
            sum += xor32(sum);
            float (*rb)[32][2] = red[it & 1];              // two buffers: one barrier per iteration
            if (g == 0) { rb[wv][r32][0] = mx; rb[wv][r32][1] = sum; }
            lds_barrier();
            if (wv == 0 && g == 0 && row < a.w) {
                float M = -INFINITY;
#pragma unroll
                for (int i = 0; i < 4; ++i) M = fmaxf(M, rb[i][r32][0]);
                const float Ms = (M == -INFINITY) ? 0.f : M;
                float L = 0.f;
#pragma unroll
                for (int i = 0; i < 4; ++i) L += rb[i][r32][1] * fast_exp2(rb[i][r32][0] - Ms);
                float* dst = a.part + (((int64_t)bh * a.w + row) * a.nkb + kb) * 2;
                dst[0] = M; dst[1] = L;
            }
        }
    }
}

// ---- merge: one wave per row; lanes stride over the key blocks, then a fixed butterfly ------------
__global__ __launch_bounds__(256) void merge_kernel(ScoreArgs a, int rows) {
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (row >= rows) return;
    const float* p = a.part + (int64_t)row * a.nkb * 2;
    float M = -INFINITY;
    for (int kb = lane; kb < a.nkb; kb += 64) M = fmaxf(M, p[2 * kb]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
    float L = 0.f;
    for (int kb = lane; kb < a.nkb; kb += 64) {
        const float m = p[2 * kb];
        if (m != -INFINITY) L += p[2 * kb + 1] * fast_exp2(m - M);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) L += __shfl_xor(L, off, 64);
    if (lane == 0) {
        a.rowstat[2 * row] = M;
        a.rowstat[2 * row + 1] = L > 0.f ? 1.0f / L : 0.f;
    }
}

// ---- pass 2: line sums ------------------------------------------------------------------------
// grid (nkb, B*Hkv), dynamic LDS: A slab [wpad][SB + 1] floats + row stats [wpad][2] + row limits [wpad] +
// the staged Q of one head.
// MODE 0: vert/vmax per head + diagonal partials (contiguous window, q_pos == NULL)
// MODE 1: vert/vmax per head + diagonals through atomics (explicit q_pos)
// MODE 2: column sums only, summed over the G heads of the KV head (retention score)
// MODE 3: no sums at all: the matrix A itself is written, [BH][w][n], zero beyond each row's position
template <typename T, int D, int MODE>
__global__ __launch_bounds__(SCORE_THREADS) void lines_kernel(ScoreArgs a) {
    using QS = QStage<T, D>;
    extern __shared__ __align__(16) unsigned char smem[];
    const int wpad = ((a.w + 31) / 32) * 32;
    float* slab = reinterpret_cast<float*>(smem);                  // [wpad][SB+1], MODE 0 only
    float* rst = slab + (MODE == 0 ? (size_t)wpad * (SB + 1) : 0); // [wpad][2], 16-byte aligned (wpad % 32 == 0)
    int32_t* ql = reinterpret_cast<int32_t*>(rst + 2 * wpad);      // [wpad] last visible key of a row, relative to the block
    unsigned char* qs = reinterpret_cast<unsigned char*>(ql + wpad);   // [wpad][D] staged queries
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, r32 = lane & 31, g = lane >> 5;
    const int kb = blockIdx.x, bk = blockIdx.y;
    const int b = bk / a.Hkv, kvh = bk % a.Hkv;
    const int64_t n = a.n;
    const T* Kg = reinterpret_cast<const T*>(a.k) + (int64_t)bk * n * D;
    const int64_t blk0 = (int64_t)kb * SB;
    const int64_t mykey = blk0 + 32 * wv + r32;
    const int klocal = 32 * wv + r32;
    const int bh0 = b * a.Hq + kvh * a.G;
    const T* Q0 = reinterpret_cast<const T*>(a.q) + (int64_t)bh0 * a.w * D;
    typename QS::Unit qu[QS::PF];
    QS::fetch(qu, Q0, a.w, wpad, tid);
    float rs_m = tid < a.w ? a.rowstat[2 * ((int64_t)bh0 * a.w + tid)] : 0.f;        // wpad <= 256 = one row per thread
    float rs_il = tid < a.w ? a.rowstat[2 * ((int64_t)bh0 * a.w + tid) + 1] : 0.f;
    Frag<T> kf[D / 16];
    load_k_frags<T, D>(kf, Kg, mykey, n, g);
    for (int i = tid; i < wpad; i += SCORE_THREADS) {
        int64_t p = (i < a.w) ? (a.q_pos ? a.q_pos[i] : n - a.w + i) : -1;
        if (p > n - 1) p = n - 1;                          // positions outside the context are clipped
        const int64_t rel = p - blk0;                      // key klocal of the block is visible to row i iff klocal <= rel
        ql[i] = rel < -1 ? -1 : (rel > SB ? SB : (int32_t)rel);
    }
    // every key of the block is visible to every row of a contiguous window (all but the last blocks)
    const bool open = a.q_pos == nullptr && blk0 + SB - 1 <= n - a.w;
    const int rgs = wpad / 32;
    float gsum = 0.f;                                              // MODE 2 accumulator over heads
    for (int gq = 0; gq < a.G; ++gq) {
        const int bh = bh0 + gq;
        const T* Qh = Q0 + (int64_t)gq * a.w * D;
        lds_barrier();                                             // slab / rst / staged Q free again
        if (tid < wpad) { rst[2 * tid] = rs_m; rst[2 * tid + 1] = rs_il; }
        QS::commit(qs, qu, Qh, a.w, wpad, tid);
        lds_barrier();
        // the next head's row statistics and queries are requested before this head's results are stored: a load
        // issued after a store would not return before the store's round trip has ended (one in-order counter)
        if (gq + 1 < a.G) {
            rs_m = tid < a.w ? a.rowstat[2 * ((int64_t)(bh + 1) * a.w + tid)] : 0.f;
            rs_il = tid < a.w ? a.rowstat[2 * ((int64_t)(bh + 1) * a.w + tid) + 1] : 0.f;
            QS::fetch(qu, Qh + (int64_t)a.w * D, a.w, wpad, tid);
        }
        float vsum = 0.f, vmx = 0.f;
        for (int rg = 0; rg < rgs; ++rg) {
            Frag<T> qf[D / 16];
            QS::frags(qf, qs, 32 * rg + r32, g);
            f32x16 s;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
            for (int c = 0; c < D / 16; ++c) mma(s, qf[c], kf[c]);   // s[r] = <q_{8(r/4)+4g+r%4}, k_lane>
            float ps = 0.f, pm = 0.f;
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int row0 = 32 * rg + 8 * q4 + 4 * g;         // registers 4*q4 .. 4*q4+3 hold rows row0 .. row0+3
                const f32x4 st0 = reinterpret_cast<const f32x4*>(rst + 2 * row0)[0];     // m, 1/l of rows row0, row0+1
                const f32x4 st1 = reinterpret_cast<const f32x4*>(rst + 2 * row0)[1];     // ... row0+2, row0+3
                const float mm[4] = {st0.x, st0.z, st1.x, st1.z}, il[4] = {st0.y, st0.w, st1.y, st1.w};
                int32_t lim[4] = {SB, SB, SB, SB};
                if (!open) {
                    typedef __attribute__((ext_vector_type(4))) int32_t i32x4;
                    const i32x4 l4 = *reinterpret_cast<const i32x4*>(ql + row0);
                    lim[0] = l4.x; lim[1] = l4.y; lim[2] = l4.z; lim[3] = l4.w;
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int r = 4 * q4 + e, row = row0 + e;
                    float p = fast_exp2(s[r] * a.scale_log2e - mm[e]) * il[e];
                    if (!open) p = (klocal <= lim[e]) ? p : 0.f;
                    ps += p;
                    pm = fmaxf(pm, p);
                    if (MODE == 0) slab[row * (SB + 1) + klocal] = p;
                    if (MODE == 3 && row < a.w && mykey < n) a.a_win[((int64_t)bh * a.w + row) * n + mykey] = p;
                    if (MODE == 1 && p > 0.f) {
                        int64_t pr = a.q_pos ? a.q_pos[row] : n - a.w + row;
                        if (pr > n - 1) pr = n - 1;
                        const int64_t o = pr - mykey;
                        atomicAdd(a.slash + (int64_t)bh * n + o, p);
                        atomicMax(reinterpret_cast<unsigned int*>(a.smax + (int64_t)bh * n + o),
                                  __builtin_bit_cast(unsigned int, p));
                    }
                }
            }
            ps += xor32(ps);
            pm = fmaxf(pm, xor32(pm));
            vsum += ps;
            vmx = fmaxf(vmx, pm);
        }
        if (MODE == 2) gsum += vsum;
        else if (MODE != 3 && g == 0 && mykey < n) {
            a.vert[(int64_t)bh * n + mykey] = vsum;
            a.vmax[(int64_t)bh * n + mykey] = vmx;
        }
        if (MODE == 0) {
            lds_barrier();
            // thread j owns diagonal o = omin + j of this slab; key_local = t + (SB-1) - j for row t
            const int64_t omin = n - a.w - (blk0 + SB - 1);
            for (int j = tid; j < SB - 1 + a.w; j += SCORE_THREADS) {
                const int64_t o = omin + j;
                if (o < 0) continue;
                float ssum = 0.f, smx = 0.f;
                const int t0 = j - (SB - 1) > 0 ? j - (SB - 1) : 0;
                const int t1 = j < a.w - 1 ? j : a.w - 1;
                // rows in ascending order, eight reads in flight; whole groups of eight need no range tests, the
                // last, shorter group adds an exact zero for a row beyond t1
                const float* dp = slab + (SB - 1) - j;             // row t of this diagonal sits at dp[t * (SB + 2)]
                int tb = t0;
                for (; tb + 7 <= t1; tb += 8) {
                    float p8[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) p8[e] = dp[(tb + e) * (SB + 2)];
#pragma unroll
                    for (int e = 0; e < 8; ++e) { ssum += p8[e]; smx = fmaxf(smx, p8[e]); }
                }
                if (tb <= t1) {
                    float p8[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) p8[e] = (tb + e <= t1) ? dp[(tb + e) * (SB + 2)] : 0.f;
#pragma unroll
                    for (int e = 0; e < 8; ++e) { ssum += p8[e]; smx = fmaxf(smx, p8[e]); }
                }
                float* dst = a.spart + (((int64_t)(kb & 1) * a.BH + bh) * n + o) * 2;
                dst[0] = ssum; dst[1] = smx;
            }
        }
    }
    if (MODE == 2 && g == 0 && mykey < n) a.gscore[(int64_t)bk * n + mykey] = gsum;
}

// ---- finish: add the two diagonal partials, reduce the total ------------------------------------
// grid (B*Hq).  Diagonal o is met by keys n-w-o .. n-1-o (clipped at 0), i.e. by key blocks
// kA = max(0, n-w-o)/SB and kB = (n-1-o)/SB, which are equal or adjacent.
constexpr int FINISH_SPLIT = 8;            // workgroups per head (a head alone is a string of load round trips)
__global__ __launch_bounds__(1024) void finish_kernel(ScoreArgs a, int contiguous) {
    __shared__ float red[1024];
    const int bh = blockIdx.x, part = blockIdx.y, tid = threadIdx.x;
    const int64_t n = a.n;
    const int64_t per = ((n + FINISH_SPLIT - 1) / FINISH_SPLIT + 1023) / 1024 * 1024;   // this workgroup's range, whole rounds of threads
    const int64_t beg = (int64_t)part * per, end = beg + per < n ? beg + per : n;
    if (contiguous) {
        for (int64_t o0 = beg + tid; o0 < end; o0 += 4 * 1024) {   // four diagonals per thread, all loads first
            float sa[4], ma[4], sb[4], mb[4]; bool two[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t o = o0 + j * 1024 < end ? o0 + j * 1024 : end - 1;
                int64_t lo = n - a.w - o; if (lo < 0) lo = 0;
                const int64_t kA = lo / SB, kB = (n - 1 - o) / SB;
                const float* pa = a.spart + (((kA & 1) * a.BH + bh) * n + o) * 2;
                const float* pb = a.spart + (((kB & 1) * a.BH + bh) * n + o) * 2;
                two[j] = kB != kA;
                sa[j] = pa[0]; ma[j] = pa[1]; sb[j] = pb[0]; mb[j] = pb[1];
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t o = o0 + j * 1024;
                if (o < end) {
                    a.slash[(int64_t)bh * n + o] = two[j] ? sa[j] + sb[j] : sa[j];      // lower key block first
                    a.smax[(int64_t)bh * n + o] = two[j] ? fmaxf(ma[j], mb[j]) : ma[j];
                }
            }
        }
    }
    // this range's share of total = sum of the column sums: per thread in index order, then a fixed tree
    float acc = 0.f;
    for (int64_t i0 = beg + tid; i0 < end; i0 += 4 * 1024) {
        float v4[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) { const int64_t i = i0 + j * 1024; v4[j] = i < end ? a.vert[(int64_t)bh * n + i] : 0.f; }
#pragma unroll
        for (int j = 0; j < 4; ++j) if (i0 + j * 1024 < end) acc += v4[j];
    }
    red[tid] = acc;
    __syncthreads();
    for (int s = 512; s > 0; s >>= 1) {
        if (tid < s) red[tid] += red[tid + s];
        __syncthreads();
    }
    if (tid == 0) a.part[(int64_t)bh * FINISH_SPLIT + part] = red[0];   // `part` is free again once merge_kernel has run
}

// total[bh] = the ranges' shares added in a fixed tree order
__global__ void total_kernel(ScoreArgs a) {
    const int bh = blockIdx.x * blockDim.x + threadIdx.x;
    if (bh >= a.BH) return;
    const float* p = a.part + (int64_t)bh * FINISH_SPLIT;
    a.total[bh] = ((p[0] + p[1]) + (p[2] + p[3])) + ((p[4] + p[5]) + (p[6] + p[7]));
}

__global__ void fill_zero_kernel(float* p, int64_t count) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0.f;
}

template <typename T, int D>
static hipError_t run_score_t(const ScoreArgs& a, int mode, hipStream_t st) {
    const dim3 grid(a.nkb, a.B * a.Hkv);
    const int wpad = ((a.w + 31) / 32) * 32;
    const size_t qbytes = (size_t)wpad * D * Elem<T>::bytes;
    hipLaunchKernelGGL((stats_kernel<T, D>), grid, dim3(SCORE_THREADS), qbytes, st, a);
    const int rows = a.BH * a.w;
    hipLaunchKernelGGL(merge_kernel, dim3((rows + 3) / 4), dim3(256), 0, st, a, rows);
    const size_t smem = (mode == 0 ? (size_t)wpad * (SB + 1) * 4 : 0) + (size_t)wpad * 8 + (size_t)wpad * 4 + qbytes;
    if (mode == 0) {
        hipLaunchKernelGGL((lines_kernel<T, D, 0>), grid, dim3(SCORE_THREADS), smem, st, a);
    } else if (mode == 1) {
        const int64_t cnt = (int64_t)a.BH * a.n;
        hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, st, a.slash, cnt);
        hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, st, a.smax, cnt);
        hipLaunchKernelGGL((lines_kernel<T, D, 1>), grid, dim3(SCORE_THREADS), smem, st, a);
    } else if (mode == 3) {
        hipLaunchKernelGGL((lines_kernel<T, D, 3>), grid, dim3(SCORE_THREADS), smem, st, a);
        return hipGetLastError();
    } else {
        hipLaunchKernelGGL((lines_kernel<T, D, 2>), grid, dim3(SCORE_THREADS), smem, st, a);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(finish_kernel, dim3(a.BH, FINISH_SPLIT), dim3(1024), 0, st, a, mode == 0 ? 1 : 0);
    hipLaunchKernelGGL(total_kernel, dim3((a.BH + 255) / 256), dim3(256), 0, st, a);
    return hipGetLastError();
}

template <typename T, int D>
static hipError_t init_score_t() {
    hipError_t e;
    if ((e = allow_full_lds(&stats_kernel<T, D>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&lines_kernel<T, D, 0>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&lines_kernel<T, D, 1>)) != hipSuccess) return e;
    if ((e = allow_full_lds(&lines_kernel<T, D, 3>)) != hipSuccess) return e;
    return allow_full_lds(&lines_kernel<T, D, 2>);
}
hipError_t init_score_kernels() {
    hipError_t e;
    if ((e = init_score_t<bf16_t, 128>()) != hipSuccess) return e;
    if ((e = init_score_t<bf16_t, 64>()) != hipSuccess) return e;
    if ((e = init_score_t<float, 128>()) != hipSuccess) return e;
    return init_score_t<float, 64>();
}

hipError_t run_score(const ScoreArgs& a, int dtype, int d, int mode, hipStream_t st) {
    if (dtype == 0 && d == 128) return run_score_t<bf16_t, 128>(a, mode, st);
    if (dtype == 0 && d == 64) return run_score_t<bf16_t, 64>(a, mode, st);
    if (dtype == 1 && d == 128) return run_score_t<float, 128>(a, mode, st);
    if (dtype == 1 && d == 64) return run_score_t<float, 64>(a, mode, st);
    return hipErrorInvalidValue;
}

// dynamic LDS of lines_kernel (the larger of the two passes)
size_t score_lines_smem(int w, int dtype, int d, int mode) {
    const int wpad = ((w + 31) / 32) * 32;
    return (mode == 0 ? (size_t)wpad * (SB + 1) * 4 : 0) + (size_t)wpad * 12 + (size_t)wpad * d * (dtype == 0 ? 2 : 4);
}

}  // namespace ls
