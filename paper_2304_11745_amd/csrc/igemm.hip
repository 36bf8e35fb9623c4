// Implicit-GEMM convolution / GEMM / attention products on CDNA4 matrix cores.
//
//   Y[m][n] = act( alpha * sum_k A[m][k] * B[n][k] + bias[n] + res[m][n] )
//
// One 256-thread workgroup (4 wavefronts of 64) owns a BM x BN output tile and walks K in blocks of
// KV 16-byte vectors per row.  Global tiles are prefetched two blocks ahead into registers, staged
// through double-buffered LDS and consumed by 32x32 MFMA tiles:
//   fp32 : v_mfma_f32_32x32x2_f32   (true fp32 multiply-accumulate)
//   bf16 : v_mfma_f32_32x32x16_bf16 (fp32 accumulate)
//
// Bit-exactness across decompositions: each output element is the ordered sum of `ksplit` slice
// accumulators; a slice accumulator is one MFMA chain that walks its k range in ascending groups of
// 32 bytes.  ksplit and the slice length are fixed per operator from its unsplit shape, so the order
// of additions never depends on the tile shape, on the position of the element inside a tile, or on
// the launched sub-range.  K tails are zero filled.  A chunk launch (Eq. 5: part of the batch, or part
// of the output channels) therefore produces exactly the bits the unsplit launch produces.
#include <hip/hip_runtime.h>
#include <string>
#include "kernels.h"

namespace gacer {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

static constexpr int THREADS = 256;
enum { LOAD_VEC = 0, LOAD_GATHER = 1, LOAD_BT = 2 };

__device__ __forceinline__ float bf16_to_f32(unsigned short v) { return __uint_as_float(((unsigned)v) << 16); }
__device__ __forceinline__ unsigned short f32_to_bf16(float f)
{
    unsigned u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (unsigned short)((u >> 16) | 0x40u);   // NaN stays NaN
    u += 0x7FFFu + ((u >> 16) & 1u);                                                     // nearest even
    return (unsigned short)(u >> 16);
}

__device__ __forceinline__ float act_apply(float v, int act)
{
    if (act == ACT_RELU) return v > 0.f ? v : 0.f;
    if (act == ACT_RELU6) return v < 0.f ? 0.f : (v > 6.f ? 6.f : v);
    if (act == ACT_GELU) return __fmul_rn(__fmul_rn(0.5f, v), __fadd_rn(1.f, erff(__fmul_rn(v, 0.70710678118654752440f))));
    return v;
}

template <int DT> struct El;
template <> struct El<DT_F32> { typedef float T; static constexpr int VEC = 4; };
template <> struct El<DT_BF16> { typedef unsigned short T; static constexpr int VEC = 8; };

// k -> (tap row r, tap col s, channel ci)
__device__ __forceinline__ void split_k(int k, int Cin, int kw, bool one_tap, int &r, int &s, int &ci)
{
    if (one_tap) { r = 0; s = 0; ci = k; return; }
    int tap = k / Cin;
    ci = k - tap * Cin;
    r = tap / kw;
    s = tap - r * kw;
}

template <typename T> __device__ __forceinline__ void store_out(T *y, int64_t o, float v);
template <> __device__ __forceinline__ void store_out<float>(float *y, int64_t o, float v) { y[o] = v; }
template <> __device__ __forceinline__ void store_out<unsigned short>(unsigned short *y, int64_t o, float v) { y[o] = f32_to_bf16(v); }
__device__ __forceinline__ float load_in(const float *p, int64_t o) { return p[o]; }
__device__ __forceinline__ float load_in(const unsigned short *p, int64_t o) { return bf16_to_f32(p[o]); }

template <int DT, int BM, int BN, int WM, int WN, int KV, int LOAD>
__global__ __launch_bounds__(THREADS) void igemm_kernel(GemmArgs a)
{
    typedef typename El<DT>::T T;
    constexpr int VEC = El<DT>::VEC;            // elements per 16-byte vector
    constexpr int BK = KV * VEC;                // elements per K block
    constexpr int ROWB = KV * 16 + 16;          // LDS bytes per tile row (16 bytes of padding)
    constexpr int RPP = THREADS / KV;           // tile rows covered by one pass of all threads
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int AV = (BM + RPP - 1) / RPP;    // 16-byte vectors per thread, A tile
    constexpr int BV = (BN + RPP - 1) / RPP;
    constexpr int NV = BN / VEC;                // LOAD_BT: n-vectors per k row of the B tile
    constexpr int BTV = (BK * NV + THREADS - 1) / THREADS;
    constexpr int BREG = LOAD == LOAD_BT ? BTV : BV;
    static_assert(WM * WN == 4 && TM >= 1 && TN >= 1, "tile shape");

    __shared__ __align__(16) unsigned char smem[2 * (BM + BN) * ROWB];
    unsigned char *As = smem, *Bs = smem + 2 * BM * ROWB;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int tiles_n = (a.n_hi - a.n_lo + BN - 1) / BN;
    const int tile_n = blockIdx.x % tiles_n, tile_m = blockIdx.x / tiles_n;
    const int m0 = a.m_lo + tile_m * BM, n0 = a.n_lo + tile_n * BN;

    const int z = blockIdx.z;
    const int zb = a.z_lo + z / a.zh, zh = z % a.zh;
    const T *xg = (const T *)a.x + zb * a.x_zb + zh * a.x_zh;
    const T *wg = (const T *)a.w + zb * a.w_zb + zh * a.w_zh;
    const int64_t y_off = zb * a.y_zb + zh * a.y_zh;

    const bool one_tap = (a.kh == 1 && a.kw == 1);
    const int HoWo = a.Ho * a.Wo;
    const int vcol = tid % KV;                  // which 16-byte vector of the row this thread moves
    const int vrow = tid / KV;

    // ---- per-thread A rows: decode output position once ----
    int64_t a_img[AV];
    int a_ih0[AV], a_iw0[AV];
    bool a_ok[AV];
#pragma unroll
    for (int i = 0; i < AV; ++i) {
        const int row = vrow + i * RPP;
        const int m = m0 + row;
        a_ok[i] = (row < BM) && (m < a.m_hi);
        const int mm = a_ok[i] ? m : a.m_lo;
        const int img = mm / HoWo, rem = mm - img * HoWo;
        const int oh = rem / a.Wo, ow = rem - oh * a.Wo;
        a_img[i] = (int64_t)img * a.x_img;
        a_ih0[i] = oh * a.stride - a.pad;
        a_iw0[i] = ow * a.stride - a.pad;
    }

    uint4 ra[2][AV], rb[2][BREG];

    auto load_global = [&](int kb, uint4 *pa, uint4 *pb) {
        const int kv = kb * BK + vcol * VEC;    // first k of this thread's vector
        if constexpr (LOAD != LOAD_GATHER) {
            int r, s, ci;
            split_k(kv, a.Cin, a.kw, one_tap, r, s, ci);
            const bool k_ok = kv < a.K;
#pragma unroll
            for (int i = 0; i < AV; ++i) {
                const int ih = a_ih0[i] + r, iw = a_iw0[i] + s;
                const bool ok = a_ok[i] && k_ok && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
                pa[i] = make_uint4(0, 0, 0, 0);
                if (ok) pa[i] = *(const uint4 *)(xg + a_img[i] + ((int64_t)ih * a.W + iw) * a.x_pix + ci);
            }
            if constexpr (LOAD == LOAD_VEC) {
#pragma unroll
                for (int i = 0; i < BV; ++i) {
                    const int row = vrow + i * RPP;
                    const int n = n0 + row;
                    pb[i] = make_uint4(0, 0, 0, 0);
                    if (row < BN && n < a.n_hi && k_ok) pb[i] = *(const uint4 *)(wg + (int64_t)n * a.w_row + kv);
                }
            } else {
                // B stored [k][n]: vectors run along n
#pragma unroll
                for (int i = 0; i < BTV; ++i) {
                    const int idx = tid + i * THREADS;
                    const int kk = idx / NV, nv = idx - kk * NV;
                    const int k = kb * BK + kk, n = n0 + nv * VEC;
                    pb[i] = make_uint4(0, 0, 0, 0);
                    if (idx < BK * NV && k < a.K && n < a.n_hi) pb[i] = *(const uint4 *)(wg + (int64_t)k * a.w_row + n);
                }
            }
        } else {
            // element-wise gather: any Cin, any alignment (stem convolutions, ragged K)
            T ea[AV][VEC], eb[BV][VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const int k = kv + e;
                int r, s, ci;
                split_k(k, a.Cin, a.kw, one_tap, r, s, ci);
                const bool k_ok = k < a.K;
#pragma unroll
                for (int i = 0; i < AV; ++i) {
                    const int ih = a_ih0[i] + r, iw = a_iw0[i] + s;
                    const bool ok = a_ok[i] && k_ok && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
                    ea[i][e] = ok ? xg[a_img[i] + ((int64_t)ih * a.W + iw) * a.x_pix + ci] : (T)0;
                }
#pragma unroll
                for (int i = 0; i < BV; ++i) {
                    const int row = vrow + i * RPP;
                    const int n = n0 + row;
                    eb[i][e] = (row < BN && n < a.n_hi && k_ok) ? wg[(int64_t)n * a.w_row + k] : (T)0;
                }
            }
#pragma unroll
            for (int i = 0; i < AV; ++i) pa[i] = *(const uint4 *)ea[i];
#pragma unroll
            for (int i = 0; i < BV; ++i) pb[i] = *(const uint4 *)eb[i];
        }
    };

    auto store_lds = [&](int buf, const uint4 *pa, const uint4 *pb) {
#pragma unroll
        for (int i = 0; i < AV; ++i) {
            const int row = vrow + i * RPP;
            if (row < BM) *(uint4 *)(As + (buf * BM + row) * ROWB + vcol * 16) = pa[i];
        }
        if constexpr (LOAD != LOAD_BT) {
#pragma unroll
            for (int i = 0; i < BV; ++i) {
                const int row = vrow + i * RPP;
                if (row < BN) *(uint4 *)(Bs + (buf * BN + row) * ROWB + vcol * 16) = pb[i];
            }
        } else {
#pragma unroll
            for (int i = 0; i < BTV; ++i) {
                const int idx = tid + i * THREADS;
                const int kk = idx / NV, nv = idx - kk * NV;
                if (idx < BK * NV) {
                    const T *e = (const T *)&pb[i];
#pragma unroll
                    for (int q = 0; q < VEC; ++q) *(T *)(Bs + (buf * BN + nv * VEC + q) * ROWB + kk * (int)sizeof(T)) = e[q];
                }
            }
        }
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int lrow = lane & 31, lhalf = lane >> 5;

    auto compute = [&](int buf) {
#pragma unroll
        for (int ks = 0; ks < KV / 2; ++ks) {
            uint4 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *(const uint4 *)(As + (buf * BM + wm * (BM / WM) + i * 32 + lrow) * ROWB + ks * 32 + lhalf * 16);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *(const uint4 *)(Bs + (buf * BN + wn * (BN / WN) + j * 32 + lrow) * ROWB + ks * 32 + lhalf * 16);
            if constexpr (DT == DT_BF16) {
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[i]),
                                                                            __builtin_bit_cast(bf16x8, fb[j]), acc[i][j], 0, 0, 0);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j) {
                            const float av = __uint_as_float(e == 0 ? fa[i].x : e == 1 ? fa[i].y : e == 2 ? fa[i].z : fa[i].w);
                            const float bv = __uint_as_float(e == 0 ? fb[j].x : e == 1 ? fb[j].y : e == 2 ? fb[j].z : fb[j].w);
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[i][j], 0, 0, 0);
                        }
            }
        }
    };

    // K range of this slice, in blocks of BK (kb_per_slice counts 64-byte blocks)
    const int nkb_all = (a.K + BK - 1) / BK;
    const int per = a.kb_per_slice / (KV / 4);
    const int slice = blockIdx.y;
    const int kb_lo = slice * per;
    const int nkb = min(nkb_all, kb_lo + per);

    // Pipeline: LDS buffer p holds block kb, register set p^1 holds block kb+1 (in flight), and the loads
    // of block kb+2 are issued into register set p before the MFMAs of block kb start.
    load_global(kb_lo, ra[0], rb[0]);
    store_lds(0, ra[0], rb[0]);
    if (kb_lo + 1 < nkb) load_global(kb_lo + 1, ra[1], rb[1]);
    __syncthreads();
    for (int kb = kb_lo; kb < nkb; kb += 2) {
        if (kb + 2 < nkb) load_global(kb + 2, ra[0], rb[0]);
        compute(0);
        if (kb + 1 < nkb) store_lds(1, ra[1], rb[1]);
        __syncthreads();
        if (kb + 1 < nkb) {
            if (kb + 3 < nkb) load_global(kb + 3, ra[1], rb[1]);
            compute(1);
            if (kb + 2 < nkb) store_lds(0, ra[0], rb[0]);
            __syncthreads();
        }
    }

    // ---- 32x32 accumulator layout: element e -> row (e/4)*8 + (lane/32)*4 + e%4, col lane%32 ----
    if (a.ksplit > 1) {
        // park the slice accumulator; splitk_finish adds the slices in order and applies the epilogue
        const int Nl = a.n_hi - a.n_lo;
        float *ws = a.ws + (int64_t)slice * (a.m_hi - a.m_lo) * Nl;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + wn * (BN / WN) + j * 32 + lrow;
            if (n >= a.n_hi) continue;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int m = m0 + wm * (BM / WM) + i * 32 + (e >> 2) * 8 + lhalf * 4 + (e & 3);
                    if (m < a.m_hi) ws[(int64_t)(m - a.m_lo) * Nl + (n - a.n_lo)] = acc[i][j][e];
                }
        }
        return;
    }
    T *yg = (T *)a.y + y_off;
    const T *rg = a.res ? (const T *)a.res + y_off : nullptr;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * (BN / WN) + j * 32 + lrow;
        if (n >= a.n_hi) continue;
        const float bias = a.bias ? a.bias[n] : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + wm * (BM / WM) + i * 32 + (e >> 2) * 8 + lhalf * 4 + (e & 3);
                if (m >= a.m_hi) continue;
                const int64_t o = (int64_t)m * a.y_row + n;
                float v = __fmaf_rn(acc[i][j][e], a.alpha, bias);
                if (rg) v = __fadd_rn(v, load_in(rg, o));
                store_out<T>(yg, o, act_apply(v, a.act));
            }
    }
}

// Second pass of a split-K operator: out = act(alpha * (s0 + s1 + ... ) + bias + res), slices added in
// ascending order.  One thread per output element of the launched sub-range, coalesced along n.
template <typename T>
__global__ __launch_bounds__(THREADS) void splitk_finish(GemmArgs a)
{
    const int Nl = a.n_hi - a.n_lo;
    const int64_t total = (int64_t)(a.m_hi - a.m_lo) * Nl;
    const int64_t idx = (int64_t)blockIdx.x * THREADS + threadIdx.x;
    if (idx >= total) return;
    const int m = a.m_lo + (int)(idx / Nl), n = a.n_lo + (int)(idx % Nl);
    float v = a.ws[idx];
    for (int q = 1; q < a.ksplit; ++q) v = __fadd_rn(v, a.ws[q * total + idx]);
    v = __fmaf_rn(v, a.alpha, a.bias ? a.bias[n] : 0.f);
    const int64_t o = (int64_t)m * a.y_row + n;
    if (a.res) v = __fadd_rn(v, load_in((const T *)a.res, o));
    store_out<T>((T *)a.y, o, act_apply(v, a.act));
}

// ------------------------------------------------------------------------------------------------
template <int DT, int BM, int BN, int WM, int WN, int KV>
static LaunchInfo go(const GemmArgs &a, hipStream_t s, bool dry, bool vec_ok)
{
    typedef typename El<DT>::T T;
    constexpr int ROWB = KV * 16 + 16;
    const int tiles_m = (a.m_hi - a.m_lo + BM - 1) / BM, tiles_n = (a.n_hi - a.n_lo + BN - 1) / BN;
    const int z = a.zb * a.zh;
    const int ks = a.b_trans ? 1 : a.ksplit;
    LaunchInfo li;
    li.workgroups = tiles_m * tiles_n * z * ks;
    li.threads = THREADS;
    li.lds_bytes = 2 * (BM + BN) * ROWB;
    const int by_lds = (160 * 1024) / li.lds_bytes;
    li.wg_per_cu = by_lds < 8 ? by_lds : 8;     // 8 wave slots per SIMD, one wave of each workgroup per SIMD
    static const std::string shape = std::string(DT == DT_BF16 ? "bf16_" : "f32_") + std::to_string(BM) + "x" + std::to_string(BN) +
                                     "x" + std::to_string(KV * El<DT>::VEC);
    static const std::string n_vec = "igemm_" + shape, n_bt = "igemm_bt_" + shape, n_gather = "igemm_gather_" + shape;
    li.kernel = a.b_trans ? n_bt.c_str() : (vec_ok ? n_vec.c_str() : n_gather.c_str());
    if (dry || li.workgroups == 0) return li;
    dim3 grid(tiles_m * tiles_n, ks, z), block(THREADS);
    if (a.b_trans)
        hipLaunchKernelGGL((igemm_kernel<DT, BM, BN, WM, WN, KV, LOAD_BT>), grid, block, 0, s, a);
    else if (vec_ok)
        hipLaunchKernelGGL((igemm_kernel<DT, BM, BN, WM, WN, KV, LOAD_VEC>), grid, block, 0, s, a);
    else
        hipLaunchKernelGGL((igemm_kernel<DT, BM, BN, WM, WN, KV, LOAD_GATHER>), grid, block, 0, s, a);
    if (ks > 1) {
        const int64_t total = (int64_t)(a.m_hi - a.m_lo) * (a.n_hi - a.n_lo);
        hipLaunchKernelGGL((splitk_finish<T>), dim3((unsigned)((total + THREADS - 1) / THREADS)), block, 0, s, a);
    }
    return li;
}

template <int DT>
static LaunchInfo pick(const GemmArgs &a, hipStream_t s, bool dry)
{
    constexpr int VEC = El<DT>::VEC;
    const bool vec_ok = (a.Cin % VEC == 0) && (a.x_pix % VEC == 0) && (a.x_img % VEC == 0) && (a.w_row % VEC == 0) &&
                        (a.x_zb % VEC == 0) && (a.x_zh % VEC == 0) && (a.w_zb % VEC == 0) && (a.w_zh % VEC == 0) &&
                        (((uintptr_t)a.x) % 16 == 0) && (((uintptr_t)a.w) % 16 == 0);
    const int M = a.m_hi - a.m_lo, N = a.n_hi - a.n_lo;
    const int64_t z = (int64_t)a.zb * a.zh * (a.b_trans ? 1 : a.ksplit);
    // Tile choice is free (it never changes the bits): narrowest N padding first, then the largest
    // tile that still gives every compute unit about two workgroups.
    auto waste = [&](int bn) { return (double)((N + bn - 1) / bn * bn) / (double)N; };
    int bn = 128;
    if (waste(64) < waste(bn) - 1e-9) bn = 64;
    if (waste(32) < waste(bn) - 1e-9) bn = 32;
    auto wgs = [&](int bm, int bnn) { return (int64_t)((M + bm - 1) / bm) * ((N + bnn - 1) / bnn) * z; };
    const int64_t want = 512;
    if (a.b_trans || a.K <= 16 * VEC) {          // short K: 64-byte blocks
        if (bn == 128 && wgs(128, 128) >= want) return go<DT, 128, 128, 2, 2, 4>(a, s, dry, vec_ok);
        if (bn >= 64) {
            if (wgs(128, 64) >= want) return go<DT, 128, 64, 2, 2, 4>(a, s, dry, vec_ok);
            return go<DT, 64, 64, 2, 2, 4>(a, s, dry, vec_ok);
        }
        return go<DT, 128, 32, 4, 1, 4>(a, s, dry, vec_ok);
    }
    if (bn == 128 && wgs(128, 128) >= want) return go<DT, 128, 128, 2, 2, 8>(a, s, dry, vec_ok);
    if (bn >= 64) {
        if (wgs(128, 64) >= want) return go<DT, 128, 64, 2, 2, 8>(a, s, dry, vec_ok);
        return go<DT, 64, 64, 2, 2, 8>(a, s, dry, vec_ok);
    }
    return go<DT, 128, 32, 4, 1, 8>(a, s, dry, vec_ok);
}

LaunchInfo launch_igemm(const GemmArgs &a, hipStream_t s, bool dry)
{
    return a.dtype == DT_BF16 ? pick<DT_BF16>(a, s, dry) : pick<DT_F32>(a, s, dry);
}

}  // namespace gacer
