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
//            64-key tiles; the cell mask is (diagonal bit | column bit), read from bitmaps in LDS.
//   phase 2: selected columns that lie in key blocks phase 1 skipped are gathered, 64 at a time,
//            into packed tiles (only the causal test remains).
// So every allowed cell is visited exactly once.  Each wave owns 32 rows and skips the 32 x 32
// sub-tiles in which none of its rows has an allowed cell.
//
// Tile products: S^T = K_tile * Q^T and O^T += V_tile^T * P^T on 32x32 MFMA, fp32 accumulation,
// online softmax in the base-2 domain.  K is staged row-major in LDS, V transposed (see vt_col).
#include "ls_device.h"
#include "ls_internal.h"

namespace ls {

constexpr int BM = 128;   // query rows per workgroup
constexpr int BN = 64;    // keys per tile
constexpr int PREFILL_THREADS = 256;

// ---------------------------------------------------------------------------------------------
// plan: per (batch, head) bitmaps of selected diagonals / columns and the per-j activity table.
//   obits, vbits : [BH][words] uint32, bit i of word i/32; words = n/32 rounded up + 8 zero words
//   tab          : [BH][tab_len] bytes, entry j+1 for j = -1 .. ; bit0 = some diagonal of
//                  [64j-63, 64j+127] is selected, bit1 = all of them are (and 64j-63 >= 0).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void plan_kernel(PlanArgs a) {
    extern __shared__ uint32_t sm[];
    const int bh = blockIdx.x;
    const int64_t n = a.n;
    const int words = a.words;
    const int tid = threadIdx.x;
    int ns = a.s_cnt[bh]; if (ns > a.cap_s) ns = a.cap_s; if (ns < 0) ns = 0;
    int nv = a.v_cnt[bh]; if (nv > a.cap_v) nv = a.cap_v; if (nv < 0) nv = 0;
    const int32_t* si = a.s_idx + (int64_t)bh * a.cap_s;
    const int32_t* vi = a.v_idx + (int64_t)bh * a.cap_v;

    // selected columns -> bitmap
    for (int i = tid; i < words; i += blockDim.x) sm[i] = 0u;
    __syncthreads();
    for (int i = tid; i < nv; i += blockDim.x) {
        const int32_t c = vi[i];
        if (c >= 0 && c < n) atomicOr(&sm[c >> 5], 1u << (c & 31));
    }
    __syncthreads();
    for (int i = tid; i < words; i += blockDim.x) a.vbits[(int64_t)bh * words + i] = sm[i];
    __syncthreads();
    // selected diagonals -> bitmap
    for (int i = tid; i < words; i += blockDim.x) sm[i] = 0u;
    __syncthreads();
    for (int i = tid; i < ns; i += blockDim.x) {
        const int32_t o = si[i];
        if (o >= 0 && o < n) atomicOr(&sm[o >> 5], 1u << (o & 31));
    }
    __syncthreads();
    for (int i = tid; i < words; i += blockDim.x) a.obits[(int64_t)bh * words + i] = sm[i];
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
    }
}

// ---------------------------------------------------------------------------------------------
// the attention kernel
// ---------------------------------------------------------------------------------------------
template <typename T, int D>
struct TileCfg {
    static constexpr int EB = Elem<T>::bytes;
    static constexpr int EPC = Elem<T>::per16;            // elements per 16-byte chunk
    static constexpr int CPR = D / EPC;                   // 16-byte chunks per K/V row
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
__device__ __forceinline__ uint32_t window32(const uint32_t* bits, int64_t base) {
    if (base <= -32) return 0u;
    if (base < 0) return bits[0] << (int)(-base);
    const int wd = (int)(base >> 5), sh = (int)(base & 31);
    const uint64_t x = (uint64_t)bits[wd] | ((uint64_t)bits[wd + 1] << 32);
    return (uint32_t)(x >> sh);
}

template <typename T, int D>
__global__ __launch_bounds__(PREFILL_THREADS) void prefill_kernel(PrefillArgs a) {
    using C = TileCfg<T, D>;
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned char* k_lds = smem;
    unsigned char* vt_lds = smem + C::K_BYTES;
    uint32_t* ob = reinterpret_cast<uint32_t*>(smem + C::K_BYTES + C::VT_BYTES);
    uint32_t* vb = ob + a.words;
    int32_t* colbuf = reinterpret_cast<int32_t*>(vb + a.words);          // 128 entries
    uint8_t* tab = reinterpret_cast<uint8_t*>(colbuf + 128);             // tab_len entries

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r32 = lane & 31, g = lane >> 5;

    // workgroup -> (head, row block); heads are spread over the 8 XCDs so that all row blocks of a
    // head run on one XCD and share its L2 for the head's K/V rows.
    int bh, qb;
    {
        const int id = blockIdx.x;
        if (a.BH % 8 == 0) {
            const int x = id & 7, s = id >> 3;
            bh = x + 8 * (s / a.nqb);
            qb = a.nqb - 1 - (s % a.nqb);
        } else {
            bh = id / a.nqb;
            qb = a.nqb - 1 - (id % a.nqb);
        }
    }
    const int b = bh / a.Hq, h = bh % a.Hq, kvh = h / a.G;
    const int64_t n = a.n, row0 = n - a.n_hat;
    const int64_t blockpos = a.pos0 + (int64_t)qb * BM;                  // multiple of 128
    const int64_t posmax = (blockpos + BM - 1 < n - 1) ? blockpos + BM - 1 : n - 1;
    const T* Kg = reinterpret_cast<const T*>(a.k) + ((int64_t)b * a.Hkv + kvh) * n * D;
    const T* Vg = reinterpret_cast<const T*>(a.v) + ((int64_t)b * a.Hkv + kvh) * n * D;
    const T* Qg = reinterpret_cast<const T*>(a.q) + (int64_t)bh * a.n_hat * D;

    // bitmaps and activity table of this head -> LDS
    for (int i = tid; i < a.words; i += PREFILL_THREADS) {
        ob[i] = a.obits[(int64_t)bh * a.words + i];
        vb[i] = a.vbits[(int64_t)bh * a.words + i];
    }
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

    f32x16 oacc[C::DBLK];
#pragma unroll
    for (int i = 0; i < C::DBLK; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[i][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float sc2 = a.scale_log2e;

    __syncthreads();

    // ---- one staged tile: masks am[0], am[1] say which of the 2 x 32 keys this lane's row may see
    auto process = [&](uint32_t am0, uint32_t am1) {
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
                const unsigned char* krow = k_lds + (32 * sub + r32) * C::K_STRIDE + 8 * g * C::EB;
#pragma unroll
                for (int c = 0; c < C::KSTEPS; ++c) {
                    Frag<T> kf;
                    load_frag(kf, krow + 16 * c * C::EB);
                    mma(s[sub], kf, qf[c]);        // s[r] = <k_{8(r/4)+4g+r%4}, q_row>
                }
            }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            const uint32_t am = sub ? am1 : am0;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kb = 8 * (r >> 2) + 4 * g + (r & 3);
                const float x = ((am >> kb) & 1u) ? s[sub][r] * sc2 : -INFINITY;
                s[sub][r] = x;
                mx = fmaxf(mx, x);
            }
        }
        mx = fmaxf(mx, xor32(mx));
        const float m_new = fmaxf(m_run, mx);
        const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
        const float corr = fast_exp2(m_run - m_safe);
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float p = fast_exp2(s[sub][r] - m_safe);
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
                    load_frag(vf, vt_lds + (32 * i + r32) * C::VT_STRIDE + (32 * sub + 16 * hh + 8 * g) * C::EB);
                    mma(oacc[i], vf, pf);          // O^T[d][row] += V^T[d][key] P^T[key][row]
                }
            }
        }
    };

    // ---- stage 64 rows of K and V into LDS; row id < 0 means "no such row" (zero fill)
    auto stage = [&](auto row_of) {
        // K: 16 lanes cover one row
        for (int id = tid; id < BN * C::CPR; id += PREFILL_THREADS) {
            const int r = id / C::CPR, c = id % C::CPR;
            const int64_t gr = row_of(r);
            f32x4 raw = {0.f, 0.f, 0.f, 0.f};
            if (gr >= 0) raw = *reinterpret_cast<const f32x4*>(reinterpret_cast<const unsigned char*>(Kg + gr * D) + 16 * c);
            *reinterpret_cast<f32x4*>(k_lds + r * C::K_STRIDE + 16 * c) = raw;
        }
        // V: one lane per key row, transposed into LDS
        {
            const int r = tid & 63, cg = tid >> 6;
            const int64_t gr = row_of(r);
            const int col = vt_col(r);
#pragma unroll
            for (int cc = 0; cc < C::CPR / 4; ++cc) {
                const int c = cg * (C::CPR / 4) + cc;
                f32x4 raw = {0.f, 0.f, 0.f, 0.f};
                if (gr >= 0) raw = *reinterpret_cast<const f32x4*>(reinterpret_cast<const unsigned char*>(Vg + gr * D) + 16 * c);
                store_vt<T>(vt_lds, C::VT_STRIDE, c * C::EPC, col, raw);
            }
        }
    };

    // ================= phase 1: key blocks crossed by a selected diagonal =================
    const int64_t jb = blockpos / BN;                      // even
    const int64_t kb_hi = posmax / BN;
    for (int64_t kb = 0; kb <= kb_hi; ++kb) {
        const int64_t j = jb - kb;                         // >= -1
        const uint8_t f = tab[j + 1];
        if (!(f & 1)) continue;
        const int64_t key0 = kb * BN;
        __syncthreads();                                   // previous tile fully consumed
        stage([&](int r) -> int64_t { const int64_t kr = key0 + r; return kr < n ? kr : -1; });
        __syncthreads();
        uint32_t am0, am1;
        if (!row_ok) { am0 = am1 = 0u; }
        else if (f & 2) { am0 = am1 = 0xFFFFFFFFu; }
        else {
            // bit i of the mask <-> key key0 + 32*sub + i <-> diagonal pos - key
            const int64_t d0 = pos - key0;                 // diagonal of the tile's first key
            am0 = __brev(window32(ob, d0 - 31));
            am1 = __brev(window32(ob, d0 - 63));
            // selected columns, limited to keys <= pos
            uint32_t c0 = vb[(key0 >> 5)], c1 = vb[(key0 >> 5) + 1];
            if (d0 < 31) c0 = (d0 < 0) ? 0u : (c0 & (0xFFFFFFFFu >> (31 - (int)d0)));
            if (d0 < 63) c1 = (d0 < 32) ? 0u : (c1 & (0xFFFFFFFFu >> (63 - (int)d0)));
            am0 |= c0; am1 |= c1;
        }
        process(am0, am1);
    }

    // ================= phase 2: selected columns outside those key blocks =================
    {
        int nv = a.v_cnt[bh]; if (nv > a.cap_v) nv = a.cap_v; if (nv < 0) nv = 0;
        const int32_t* vi = a.v_idx + (int64_t)bh * a.cap_v;
        int cur = 0, fill = 0;
        bool more = nv > 0;
        while (true) {
            // refill the column buffer (every wave computes the same thing; wave 0 writes)
            while (more && fill < BN) {
                const int i = cur + lane;
                int32_t col = (i < nv) ? vi[i] : 0x7FFFFFFF;
                const bool inrange = (i < nv) && (col >= 0) && ((int64_t)col <= posmax);
                bool keep = false;
                if (inrange) keep = !(tab[jb - (col >> 6) + 1] & 1);
                const uint64_t km = __ballot(keep);
                if (keep && wv == 0) colbuf[fill + __popcll(km & ((1ull << lane) - 1ull))] = col;
                fill += __popcll(km);
                cur += 64;
                // the list is ascending: once an entry lies beyond the block's last row, nothing follows
                const uint64_t beyond = __ballot((i < nv) && ((int64_t)col > posmax));
                if (cur >= nv || beyond != 0ull) more = false;
            }
            if (fill == 0) break;
            const int cnt = fill < BN ? fill : BN;
            __syncthreads();                               // colbuf visible; previous tile consumed
            stage([&](int r) -> int64_t { return r < cnt ? (int64_t)colbuf[r] : -1; });
            // causal mask: columns are ascending, so the visible ones form a prefix
            uint32_t am0 = 0u, am1 = 0u;
            if (row_ok) {
                if ((int64_t)colbuf[cnt - 1] <= pos) {
                    am0 = cnt >= 32 ? 0xFFFFFFFFu : ((1u << cnt) - 1u);
                    am1 = cnt >= 64 ? 0xFFFFFFFFu : (cnt > 32 ? ((1u << (cnt - 32)) - 1u) : 0u);
                } else {
                    for (int i = 0; i < cnt; ++i) {
                        if ((int64_t)colbuf[i] <= pos) { if (i < 32) am0 |= 1u << i; else am1 |= 1u << (i - 32); }
                    }
                }
            }
            __syncthreads();
            process(am0, am1);
            __syncthreads();                               // all waves done with colbuf[0..63] and the tile
            if (fill > BN) {
                int32_t t = 0;
                if (wv == 0 && lane < fill - BN) t = colbuf[BN + lane];
                __builtin_amdgcn_wave_barrier();
                if (wv == 0 && lane < fill - BN) colbuf[lane] = t;
                fill -= BN;
            } else fill = 0;
        }
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
                l_tot > 0.f ? (m_run + log2f(l_tot)) * 0.69314718055994531f : -INFINITY;
    }
}

template <typename T, int D>
static hipError_t launch_prefill_t(const PrefillArgs& a, hipStream_t st) {
    using C = TileCfg<T, D>;
    const size_t smem = C::K_BYTES + C::VT_BYTES + 2 * (size_t)a.words * 4 + 128 * 4 + (size_t)a.tab_len;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_kernel<T, D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((prefill_kernel<T, D>), dim3(a.BH * a.nqb), dim3(PREFILL_THREADS), smem, st, a);
    return hipGetLastError();
}

size_t prefill_smem_bytes(int dtype, int d, int words, int tab_len) {
    size_t tiles = 0;
    if (dtype == 0 && d == 128) tiles = TileCfg<bf16_t, 128>::K_BYTES + TileCfg<bf16_t, 128>::VT_BYTES;
    else if (dtype == 0 && d == 64) tiles = TileCfg<bf16_t, 64>::K_BYTES + TileCfg<bf16_t, 64>::VT_BYTES;
    else if (dtype == 1 && d == 128) tiles = TileCfg<float, 128>::K_BYTES + TileCfg<float, 128>::VT_BYTES;
    else tiles = TileCfg<float, 64>::K_BYTES + TileCfg<float, 64>::VT_BYTES;
    return tiles + 2 * (size_t)words * 4 + 128 * 4 + (size_t)tab_len;
}

hipError_t launch_plan(const PlanArgs& a, int BH, hipStream_t st) {
    const size_t smem = (size_t)a.words * 4;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&plan_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(plan_kernel, dim3(BH), dim3(1024), smem, st, a);
    return hipGetLastError();
}

hipError_t launch_prefill(const PrefillArgs& a, int dtype, int d, hipStream_t st) {
    if (dtype == 0 && d == 128) return launch_prefill_t<bf16_t, 128>(a, st);
    if (dtype == 0 && d == 64) return launch_prefill_t<bf16_t, 64>(a, st);
    if (dtype == 1 && d == 128) return launch_prefill_t<float, 128>(a, st);
    if (dtype == 1 && d == 64) return launch_prefill_t<float, 64>(a, st);
    return hipErrorInvalidValue;
}

}  // namespace ls
