// Decode step over a compressed cache (Alg. 3, the Decoding step; Sec. 5.2): the newest token's query
// attends over the entries its KV head retained at the last retention step followed by the tokens
// generated since (Alg. 3 adds every generated token to the retained set), all of them visible:
//     out = softmax(scale * q [K_c; K_t]^T) [V_c; V_t].
//
// The step reads every retained K and V row once and does 4 d FLOP per (query head, key): it is bound
// by HBM bandwidth.  The G query heads of a KV head are the columns of one 32x32 MFMA tile product, so
// the rows are read once for all of them:
//   decode_partial_kernel  grid (splits, B*Hkv).  The keys of a KV head are cut into `splits` chunks;
//                          in a workgroup each of the 4 waves takes 32-key tiles of the chunk.  K
//                          fragments come straight from global memory (a key per lane), S^T = K Q^T,
//                          online softmax per head in a lane, P -> bf16, O^T += V^T P^T with the V^T
//                          fragments read transposed from a wave-private, swizzled LDS copy of the
//                          32 V rows that a global -> LDS transfer filled.  The waves' partial results
//                          (reference, normaliser, unnormalised output) are merged through LDS and
//                          written per split.
//   decode_combine_kernel  grid (B*Hq): merges the splits, normalises, writes out and lse.
// bf16 only (the transpose read is 16-bit).
#include "ls_device.h"
#include "ls_internal.h"

namespace ls {

constexpr int DEC_THREADS = 256;
constexpr int DEC_TILE = 32;                   // keys per wave tile

template <int D>
struct DecCfg {
    static_assert(D == 128 || D == 64, "head dimension");
    static constexpr int RB = D * 2;                      // bytes per row
    static constexpr int DS = RB / 16;                    // 16-byte slots per row
    static constexpr int RPI = 64 / DS;                   // rows per transfer instruction
    static constexpr int NIV = DEC_TILE / RPI;            // transfers per V tile
    static constexpr int V_BYTES = DEC_TILE * RB;         // one wave's V stage
    static constexpr int KSTEPS = D / 16, DBLK = D / 32;
    // slot swizzle of the staged V rows (XOR on the 16-byte slot index): makes the transpose reads touch
    // every LDS bank once per pass
    __device__ static constexpr int vswz(int row) { return D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2); }
};

template <int D>
__global__ __launch_bounds__(DEC_THREADS, 2) void decode_partial_kernel(DecodeArgs a) {
    using C = DecCfg<D>;
    using T = bf16_t;
    extern __shared__ __align__(16) unsigned char dec_lds[];   // 4 V stages; later the waves' partial results
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r32 = lane & 31, g = lane >> 5;
    const int split = blockIdx.x, bk = blockIdx.y;
    const int b = bk / a.Hkv, kvh = bk % a.Hkv;
    const int G = a.G;
    int nc = a.cnt ? a.cnt[bk] : a.cap;
    if (nc < 0) nc = 0;
    if (nc > a.cap) nc = a.cap;
    nc = __builtin_amdgcn_readfirstlane(nc);
    const int L = nc + a.T;                                    // keys of this KV head
    const int k0 = split * a.chunk;
    const int k1 = k0 + a.chunk < L ? k0 + a.chunk : L;
    const unsigned char* kc = reinterpret_cast<const unsigned char*>(a.kc) + (int64_t)bk * a.cap * C::RB;
    const unsigned char* vc = reinterpret_cast<const unsigned char*>(a.vc) + (int64_t)bk * a.cap * C::RB;
    const unsigned char* kt = reinterpret_cast<const unsigned char*>(a.kt) + (int64_t)bk * a.T * C::RB;
    const unsigned char* vt = reinterpret_cast<const unsigned char*>(a.vt) + (int64_t)bk * a.T * C::RB;
    auto row_of = [&](const unsigned char* retained, const unsigned char* tail, int key) -> const unsigned char* {
        return key < nc ? retained + (int64_t)key * C::RB : tail + (int64_t)(key - nc) * C::RB;
    };

    // query fragments: head r32 of the group is column r32 of the tile product
    Frag<T> qf[C::KSTEPS];
    if (r32 < G) {
        const T* qrow = reinterpret_cast<const T*>(a.q) + ((int64_t)b * a.Hq + kvh * G + r32) * D;
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
    float m_run = -INFINITY, l_run = 0.f;                      // m_run in raw logit units
    const float sc2 = a.scale_log2e;

    unsigned char* stage = dec_lds + wv * C::V_BYTES;
    const uint32_t stage_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)stage;
    // transfers: this lane fills slot sl of tile row RPI*q + lane / DS and fetches the chunk the swizzle assigns to it
    const int trow = lane / C::DS, sl = lane % C::DS;
    // transpose reads: key 4g + L16/4 (+8, +16 q4), 64-byte block i
    int vaddr[C::DBLK];
    {
        const int L16 = lane & 15, beta = (lane >> 4) & 1;
        const int lrow = 4 * g + (L16 >> 2);
        const int y = C::vswz(lrow) >> 2;
#pragma unroll
        for (int i = 0; i < C::DBLK; ++i) vaddr[i] = lrow * C::RB + 64 * (i ^ y) + 32 * beta + 8 * (L16 & 3);
    }

    for (int t0 = k0 + DEC_TILE * wv; t0 < k1; t0 += 4 * DEC_TILE) {
        // V rows of the tile -> LDS (rows past the chunk re-load its last row; their keys are masked)
#pragma unroll
        for (int q = 0; q < C::NIV; ++q) {
            const int row = C::RPI * q + trow;
            int key = t0 + row; if (key > k1 - 1) key = k1 - 1;
            dma16(row_of(vc, vt, key) + 16 * (sl ^ C::vswz(row)), stage_lds + (uint32_t)(q * 1024));
        }
        // K fragments of this lane's key, S^T = K Q^T
        int mykey = t0 + r32; if (mykey > k1 - 1) mykey = k1 - 1;
        const unsigned char* krow = row_of(kc, kt, mykey);
        Frag<T> kf[C::KSTEPS];
#pragma unroll
        for (int c = 0; c < C::KSTEPS; ++c) load_frag(kf[c], krow + 32 * c + 16 * g);
        f32x16 s = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < C::KSTEPS; ++c) mma(s, kf[c], qf[c]);      // s[r] = <k_{8(r/4)+4g+r%4}, q_head>
        const int left = k1 - t0;                                      // keys of the tile that exist
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = 8 * (r >> 2) + 4 * g + (r & 3);
            const float x = key < left ? s[r] : -INFINITY;
            s[r] = x;
            mx = fmaxf(mx, x);
        }
        mx = fmaxf(mx, xor32(mx));
        const float m_new = fmaxf(m_run, mx);                          // finite: the tile holds at least one key
        const float corr = fast_exp2((m_run - m_new) * sc2);
        const float mneg = -m_new * sc2;
        m_run = m_new;
        float ps = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float p = fast_exp2(__builtin_fmaf(s[r], sc2, mneg));
            s[r] = p;
            ps += p;
        }
        l_run = l_run * corr + ps;
        if (__ballot(corr != 1.0f) != 0ull) {
#pragma unroll
            for (int i = 0; i < C::DBLK; ++i)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[i][r] *= corr;
        }
        wait_transfers();                                              // the V rows have landed (same wave reads them)
#pragma unroll
        for (int q4 = 0; q4 < 2; ++q4) {
            float pv[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) pv[e] = s[8 * q4 + e];
            Frag<T> pf;
            pack_frag(pf, pv);
#pragma unroll
            for (int i = 0; i < C::DBLK; ++i) {
                Frag<T> vf;
                const unsigned char* va = stage + vaddr[i] + 16 * q4 * C::RB;
                load_frag_tr(vf, va, va + 8 * C::RB);
                mma(oacc[i], vf, pf);
            }
        }
    }

    // ---- merge the four waves through LDS: part[wv][head][D + 2] (output, reference, normaliser)
    const float l_tot = l_run + xor32(l_run);
    __syncthreads();                                                   // every wave is done with its V stage
    float* part = reinterpret_cast<float*>(dec_lds);
    constexpr int PS = D + 2;
    if (r32 < G) {
        float* mine = part + ((int64_t)wv * G + r32) * PS;
#pragma unroll
        for (int i = 0; i < C::DBLK; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) mine[32 * i + 8 * (r >> 2) + 4 * g + (r & 3)] = oacc[i][r];
        if (g == 0) { mine[D] = m_run; mine[D + 1] = l_tot; }
    }
    __syncthreads();
    for (int idx = tid; idx < G * PS; idx += DEC_THREADS) {
        const int head = idx / PS, dd = idx % PS;
        float m = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) m = fmaxf(m, part[((int64_t)w * G + head) * PS + D]);
        float acc = 0.f;
        if (dd != D) {                                                 // output element or normaliser: scaled sum over the waves
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float mw = part[((int64_t)w * G + head) * PS + D];
                if (mw > -INFINITY) acc += part[((int64_t)w * G + head) * PS + dd] * fast_exp2((mw - m) * sc2);
            }
        }
        float* dst = a.part + (((int64_t)bk * a.nsplit + split) * G + head) * PS;
        dst[dd] = dd == D ? m : acc;
    }
}

// grid (B*Hq), D threads: thread dd owns one output element.
template <int D>
__global__ __launch_bounds__(D) void decode_combine_kernel(DecodeArgs a) {
    constexpr int PS = D + 2;
    const int bh = blockIdx.x, dd = threadIdx.x;
    const int b = bh / a.Hq, h = bh % a.Hq, kvh = h / a.G, hh = h % a.G;
    const int bk = b * a.Hkv + kvh;
    const float* base = a.part + ((int64_t)bk * a.nsplit * a.G + hh) * PS;
    const int64_t stride = (int64_t)a.G * PS;
    float m = -INFINITY;
    for (int s = 0; s < a.nsplit; ++s) m = fmaxf(m, base[s * stride + D]);
    float o = 0.f, l = 0.f;
    for (int s = 0; s < a.nsplit; ++s) {
        const float ms = base[s * stride + D];
        if (ms > -INFINITY) {
            const float wgt = fast_exp2((ms - m) * a.scale_log2e);
            o += base[s * stride + dd] * wgt;
            l += base[s * stride + D + 1] * wgt;
        }
    }
    bf16_t* out = reinterpret_cast<bf16_t*>(a.out) + (int64_t)bh * D;
    bf16_t r; r.bits = f2bf(l > 0.f ? o / l : 0.f);
    out[dd] = r;
    if (a.lse && dd == 0) a.lse[bh] = l > 0.f ? (m * a.scale_log2e + log2f(l)) * 0.69314718055994531f : -INFINITY;
}

size_t decode_smem_bytes(int d, int G) {
    const size_t stages = 4 * (size_t)DEC_TILE * d * 2;
    const size_t merge = 4 * (size_t)G * (d + 2) * 4;
    return stages > merge ? stages : merge;
}

template <int D>
static hipError_t run_decode_t(const DecodeArgs& a, hipStream_t st) {
    const size_t smem = decode_smem_bytes(D, a.G);
    hipLaunchKernelGGL((decode_partial_kernel<D>), dim3(a.nsplit, a.B * a.Hkv), dim3(DEC_THREADS), smem, st, a);
    hipLaunchKernelGGL((decode_combine_kernel<D>), dim3(a.B * a.Hq), dim3(D), 0, st, a);
    return hipGetLastError();
}

hipError_t init_decode_kernels() {
    const hipError_t e = allow_full_lds(&decode_partial_kernel<128>);
    return e != hipSuccess ? e : allow_full_lds(&decode_partial_kernel<64>);
}

hipError_t run_decode(const DecodeArgs& a, int d, hipStream_t st) {
    if (d == 128) return run_decode_t<128>(a, st);
    if (d == 64) return run_decode_t<64>(a, st);
    return hipErrorInvalidValue;
}

}  // namespace ls
