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
#include "device_util.h"
#include "kernels.h"

namespace gacer {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

static constexpr int THREADS = 256;
enum { LOAD_VEC = 0, LOAD_GATHER = 1, LOAD_BT = 2, LOAD_TAPS = 3, LOAD_AFFINE = 4 };

__device__ __forceinline__ float bf16_to_f32(unsigned short v) { return __uint_as_float(((unsigned)v) << 16); }
__device__ __forceinline__ unsigned short f32_to_bf16(float f)     // round to nearest even (hardware conversion)
{
    return __builtin_bit_cast(unsigned short, (__bf16)f);
}

// exact (erf) GELU; kept out of line so that the unrolled epilogues stay small
__device__ __attribute__((noinline)) float gelu_erf(float v)
{
    return __fmul_rn(__fmul_rn(0.5f, v), __fadd_rn(1.f, erff(__fmul_rn(v, 0.70710678118654752440f))));
}

__device__ __forceinline__ float gelu_erf_inl(float v)
{
    return __fmul_rn(__fmul_rn(0.5f, v), __fadd_rn(1.f, erff(__fmul_rn(v, 0.70710678118654752440f))));
}

__device__ __forceinline__ float act_apply(float v, int act)
{
    if (act == ACT_RELU) return __builtin_fmaxf(v, 0.f);
    if (act == ACT_RELU6) return __builtin_amdgcn_fmed3f(v, 0.f, 6.f);
    if (act == ACT_GELU) return gelu_erf(v);
    if (act == ACT_HSWISH || act == ACT_HSIGMOID) return hard_act(v, act);
    return v;
}

template <int DT> struct El;
template <> struct El<DT_F32> { typedef float T; static constexpr int VEC = 4; };
template <> struct El<DT_BF16> { typedef unsigned short T; static constexpr int VEC = 8; };

template <typename T> __device__ __forceinline__ void store_out(T *y, int64_t o, float v);
template <> __device__ __forceinline__ void store_out<float>(float *y, int64_t o, float v) { y[o] = v; }
template <> __device__ __forceinline__ void store_out<unsigned short>(unsigned short *y, int64_t o, float v) { y[o] = f32_to_bf16(v); }
__device__ __forceinline__ float load_in(const float *p, int64_t o) { return p[o]; }
__device__ __forceinline__ float load_in(const unsigned short *p, int64_t o) { return bf16_to_f32(p[o]); }

// two floats -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32)
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi)
{
    const f32x2 f = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(f, bf16x2));
}

// Activation of EV values; `act` is uniform over the launch, so the branch is taken once per vector.
template <int EV> __device__ __forceinline__ void act_vec(float *v, int act)
{
    if (act == ACT_RELU) {                        // clamps as single v_max / v_med3 instructions, no divergent branches
#pragma unroll
        for (int q = 0; q < EV; ++q) v[q] = __builtin_fmaxf(v[q], 0.f);
    } else if (act == ACT_RELU6) {
#pragma unroll
        for (int q = 0; q < EV; ++q) v[q] = __builtin_amdgcn_fmed3f(v[q], 0.f, 6.f);
    } else if (act == ACT_GELU) {
#pragma unroll
        for (int q = 0; q < EV; ++q) v[q] = gelu_erf(v[q]);
    } else if (act == ACT_HSWISH || act == ACT_HSIGMOID) {
#pragma unroll
        for (int q = 0; q < EV; ++q) v[q] = hard_act(v[q], act);
    }
}

// Epilogue of EV consecutive output channels of one row, all inside the launched range and 16-byte aligned:
// y = act(alpha * v + bias + res).  Bias and residual arrive preloaded (their loads are issued before the accumulators
// are turned through LDS, so that no global round trip sits between the last MFMA and the output store).
template <int DT>
__device__ __forceinline__ void finish_vec(const GemmArgs &a, float *v, const float *bv, bool has_res, const uint4 &rv,
                                           typename El<DT>::T *yg, int64_t o)
{
    constexpr int EV = DT == DT_BF16 ? 8 : 4;
#pragma unroll
    for (int q = 0; q < EV; ++q) v[q] = __fmaf_rn(v[q], a.alpha, bv[q]);
    if (has_res) {
        const unsigned rw[4] = {rv.x, rv.y, rv.z, rv.w};
        if constexpr (DT == DT_BF16) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                v[2 * q] = __fadd_rn(v[2 * q], __uint_as_float(rw[q] << 16));
                v[2 * q + 1] = __fadd_rn(v[2 * q + 1], __uint_as_float(rw[q] & 0xFFFF0000u));
            }
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = __fadd_rn(v[q], __uint_as_float(rw[q]));
        }
    }
    act_vec<EV>(v, a.act);
    if constexpr (DT == DT_BF16)
        *(uint4 *)(yg + o) = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]));
    else
        *(float4 *)(yg + o) = make_float4(v[0], v[1], v[2], v[3]);
}

// bias of EV consecutive channels (zeros without a bias pointer); n is a multiple of 4 and the pointer 16-byte aligned
template <int EV> __device__ __forceinline__ void load_bias_vec(const float *bias, int n, bool ok, float *bv)
{
#pragma unroll
    for (int q = 0; q < EV; ++q) bv[q] = 0.f;
    if (bias && ok) {
#pragma unroll
        for (int q = 0; q < EV; q += 4) {
            const float4 b4 = *(const float4 *)(bias + n + q);
            bv[q] = b4.x; bv[q + 1] = b4.y; bv[q + 2] = b4.z; bv[q + 3] = b4.w;
        }
    }
}

// Ragged or unaligned tail: element by element (rare: odd channel counts, unaligned channel chunks).
template <int DT>
__device__ __noinline__ void finish_one(float v, float alpha, const float *bias, int act, const typename El<DT>::T *rg,
                                        typename El<DT>::T *yg, int64_t o, int n, int n_hi)
{
    if (n >= n_hi) return;
    float t = __fmaf_rn(v, alpha, bias ? bias[n] : 0.f);
    if (rg) t = __fadd_rn(t, load_in(rg, o));
    // leaf function (no nested call, hence no stack): the activation is expanded in place
    if (act == ACT_RELU) t = __builtin_fmaxf(t, 0.f);
    else if (act == ACT_RELU6) t = __builtin_amdgcn_fmed3f(t, 0.f, 6.f);
    else if (act == ACT_GELU) t = gelu_erf_inl(t);
    else if (act == ACT_HSWISH || act == ACT_HSIGMOID) t = hard_act(t, act);
    store_out<typename El<DT>::T>(yg, o, t);
}
template <int DT>
__device__ __forceinline__ void finish_scalar(const GemmArgs &a, const float *v, const typename El<DT>::T *rg, typename El<DT>::T *yg, int64_t o, int n)
{
    constexpr int EV = DT == DT_BF16 ? 8 : 4;
#pragma unroll
    for (int q = 0; q < EV; ++q) finish_one<DT>(v[q], a.alpha, a.bias, a.act, rg, yg, o + q, n + q, a.n_hi);
}

// ---- epilogue shared by the tiled kernels ----
// MFMA leaves element e of a 32x32 tile at row (e/4)*8 + (lane/32)*4 + e%4, column lane%32.  Each wave
// turns its tiles through a private LDS patch (`stage`, 32 rows of 36 floats) so that a lane owns EV consecutive
// output channels of one row: residual loads and output stores are then 16-byte vectors along the contiguous axis.
template <int DT, int BM, int BN, int WM, int WN>
__device__ __forceinline__ void igemm_epilogue(const GemmArgs &a, f32x16 (&acc)[BM / WM / 32][BN / WN / 32], float *stage, int m0, int n0,
                                               int wm, int wn, int lane, int slice, int64_t y_off)
{
    typedef typename El<DT>::T T;
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    const int lrow = lane & 31, lhalf = lane >> 5;
    constexpr int EV = DT == DT_BF16 ? 8 : 4;          // outputs per lane and group
    constexpr int LPR = 32 / EV;                        // lanes per tile row
    constexpr int GROUPS = 16 / EV;                     // row groups per lane
    constexpr int SROW = 36;                            // floats per staged row (16-byte aligned, padded)
    const bool split = a.ksplit > 1;
    const int Nl = a.n_hi - a.n_lo;
    float *ws = split ? a.ws + (int64_t)slice * (a.m_hi - a.m_lo) * Nl : nullptr;
    T *yg = (T *)a.y + y_off;
    const T *rg = a.res ? (const T *)a.res + y_off : nullptr;
    const bool vec_out = split ? (Nl % 4 == 0 && (((uintptr_t)a.ws) & 15) == 0)
                               : (a.y_row % EV == 0 && a.n_lo % EV == 0 && (y_off % EV) == 0 && (((uintptr_t)a.y) & 15) == 0 &&
                                  (((uintptr_t)a.res) & 15) == 0 && (((uintptr_t)a.bias) & 15) == 0);
    const int erow = lane / LPR, ecol = (lane % LPR) * EV;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = n0 + wn * (BN / WN) + j * 32 + ecol;
            const bool n_vec = vec_out && n + EV <= a.n_hi;
            // bias and residual loads first, then the LDS turn: one global round trip per tile, overlapped with the turn
            float bv[EV];
            load_bias_vec<EV>(a.bias, n, !split && n_vec, bv);
            uint4 rv[GROUPS];
#pragma unroll
            for (int g = 0; g < GROUPS; ++g) {
                const int m = m0 + wm * (BM / WM) + i * 32 + erow + g * (64 / LPR);
                rv[g] = make_uint4(0u, 0u, 0u, 0u);
                if (!split && rg && n_vec && m < a.m_hi) rv[g] = *(const uint4 *)(rg + (int64_t)m * a.y_row + n);
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) stage[((e >> 2) * 8 + lhalf * 4 + (e & 3)) * SROW + lrow] = acc[i][j][e];
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int g = 0; g < GROUPS; ++g) {
                const int row = erow + g * (64 / LPR);
                const int m = m0 + wm * (BM / WM) + i * 32 + row;
                float v[EV];
#pragma unroll
                for (int q = 0; q < EV; q += 4) {
                    const float4 t4 = *(const float4 *)(stage + row * SROW + ecol + q);
                    v[q] = t4.x; v[q + 1] = t4.y; v[q + 2] = t4.z; v[q + 3] = t4.w;
                }
                if (m >= a.m_hi || n >= a.n_hi) continue;
                if (split) {
                    float *p = ws + (int64_t)(m - a.m_lo) * Nl + (n - a.n_lo);
                    if (vec_out && n + EV <= a.n_hi) {
#pragma unroll
                        for (int q = 0; q < EV; q += 4) *(float4 *)(p + q) = make_float4(v[q], v[q + 1], v[q + 2], v[q + 3]);
                    } else {
#pragma unroll
                        for (int q = 0; q < EV; ++q)
                            if (n + q < a.n_hi) p[q] = v[q];
                    }
                    continue;
                }
                const int64_t o = (int64_t)m * a.y_row + n;
                if (n_vec) finish_vec<DT>(a, v, bv, rg != nullptr, rv[g], yg, o);
                else finish_scalar<DT>(a, v, rg, yg, o, n);
            }
            __builtin_amdgcn_wave_barrier();
        }
}

// Workgroups are handed to the 8 XCDs round-robin by their index, and each XCD has its own L2.  Neighbouring tiles share
// operand rows (the halo of a k x k window, the A rows of tiles that differ only in n, the B rows of tiles that differ
// only in m), so tile numbers are dealt such that every XCD works on one contiguous run of them: workgroup b -> XCD
// b % 8 -> the (b / 8)-th tile of that XCD's run.  Whether the runs are bands of m or bands of n is tile_order()'s choice.
__device__ __forceinline__ int xcd_contiguous(int b, int n)
{
    const int q = n >> 3, r = n & 7, x = b & 7;
    return __builtin_amdgcn_readfirstlane(x * q + min(x, r) + (b >> 3));
}

// One validity bit per tap (bit r * kw + q) of a window whose origin is (ih0, iw0): rows and columns are tested once each.
__device__ __forceinline__ unsigned tap_mask(int ih0, int iw0, int H, int W, int kh, int kw)
{
    unsigned cols = 0, tm = 0;
    for (int q = 0; q < kw; ++q) cols |= (unsigned)(iw0 + q >= 0 && iw0 + q < W) << q;
    for (int r = 0; r < kh; ++r) tm |= (ih0 + r >= 0 && ih0 + r < H) ? cols << (r * kw) : 0u;
    return tm;
}

template <int DT, int BM, int BN, int WM, int WN, int KV, int LOAD>
__global__ __launch_bounds__(THREADS) void igemm_kernel(GemmArgs a)
{
    typedef typename El<DT>::T T;
    constexpr int VEC = El<DT>::VEC;            // elements per 16-byte vector
    constexpr int ESZ = (int)sizeof(T);
    constexpr int BK = KV * VEC;                // elements per K block
    constexpr int ROWB = KV * 16 + 16;          // LDS bytes per tile row (16 bytes of padding)
    constexpr int RPP = THREADS / KV;           // tile rows covered by one pass of all threads
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int AV = (BM + RPP - 1) / RPP;    // 16-byte vectors per thread, A tile
    constexpr int BV = (BN + RPP - 1) / RPP;
    constexpr int NV = BN / VEC;                // LOAD_BT: n-vectors per k row of the B tile
    constexpr int BTV = (BK * NV + THREADS - 1) / THREADS;
    constexpr int BREG = LOAD == LOAD_BT ? BTV : BV;
    constexpr bool TAPS = (LOAD == LOAD_TAPS);  // k walks (tap row, tap col, channel); otherwise one tap
    static_assert(WM * WN == 4 && TM >= 1 && TN >= 1, "tile shape");

    __shared__ __align__(16) unsigned char smem[2 * (BM + BN) * ROWB];
    unsigned char *As = smem, *Bs = smem + 2 * BM * ROWB;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int tile = xcd_contiguous((int)blockIdx.x, (int)gridDim.x);
    const int by_m = div_by(tile, a.div_tiles_m), by_n = div_by(tile, a.div_tiles_n);
    const int tile_m = __builtin_amdgcn_readfirstlane(a.n_major ? tile - by_m * a.tiles_m : by_n);
    const int tile_n = __builtin_amdgcn_readfirstlane(a.n_major ? by_m : tile - by_n * a.tiles_n);
    const int m0 = a.m_lo + tile_m * BM, n0 = a.n_lo + tile_n * BN;

    const int z = blockIdx.z;
    const int zq = __builtin_amdgcn_readfirstlane(div_by(z, a.div_zh));
    const int zb = a.z_lo + zq, zh = z - zq * a.zh;
    const int64_t x_zoff = zb * a.x_zb + zh * a.x_zh, w_zoff = zb * a.w_zb + zh * a.w_zh;
    const __amdgpu_buffer_rsrc_t xr = make_rsrc((const T *)a.x + x_zoff, a.x_bytes - x_zoff * ESZ);
    const __amdgpu_buffer_rsrc_t wr = make_rsrc((const T *)a.w + w_zoff, a.w_bytes - w_zoff * ESZ);
    const int64_t y_off = zb * a.y_zb + zh * a.y_zh;

    const int HoWo = a.Ho * a.Wo;
    const int vcol = tid % KV;                  // which 16-byte vector of the row this thread moves
    const int vrow = tid / KV;

    // ---- per-thread A rows: byte offset of the window origin (or OOB) and validity masks of its taps ----
    unsigned a_off[AV], a_hm[AV], a_wm[AV];
#pragma unroll
    for (int i = 0; i < AV; ++i) {
        const int row = vrow + i * RPP;
        const int m = m0 + row;
        const bool ok = (row < BM) && (m < a.m_hi);
        const int mm = ok ? m : a.m_lo;
        const int img = div_by(mm, a.div_howo), rem = mm - img * HoWo;
        const int oh = div_by(rem, a.div_wo), ow = rem - oh * a.Wo;
        const int ih0 = oh * a.stride - a.pad, iw0 = ow * a.stride - a.pad;
        const int64_t e0 = (int64_t)img * a.x_img + ((int64_t)ih0 * a.W + iw0) * a.x_pix;   // may be negative at the border
        a_off[i] = ok ? (unsigned)(int)(e0 * ESZ) : OOB;
        unsigned hm = 0, wmk = 0;
        for (int r = 0; r < a.kh; ++r) hm |= (unsigned)(ih0 + r >= 0 && ih0 + r < a.H) << r;
        for (int q = 0; q < a.kw; ++q) wmk |= (unsigned)(iw0 + q >= 0 && iw0 + q < a.W) << q;
        a_hm[i] = ok ? hm : 0u;
        a_wm[i] = wmk;
        if constexpr (TAPS)                     // one validity bit per tap (kh*kw <= 31 on this path): bit r*kw + q
            a_hm[i] = ok ? tap_mask(ih0, iw0, a.H, a.W, a.kh, a.kw) : 0u;
    }
    // ---- per-thread B rows: byte offset of the weight row, and whether the row exists ----
    unsigned b_off[BV];
    bool b_ok[BV];
#pragma unroll
    for (int i = 0; i < BV; ++i) {
        const int row = vrow + i * RPP;
        const int n = n0 + row;
        b_ok[i] = row < BN && n < a.n_hi;
        b_off[i] = b_ok[i] ? (unsigned)((int64_t)n * a.w_row * ESZ) : 0u;
    }

    // K range of this slice, in blocks of BK (kb_per_slice counts 64-byte blocks)
    const int nkb_all = (a.K + BK - 1) / BK;
    const int per = a.kb_per_slice / (KV / 4);
    const int slice = blockIdx.y;
    const int kb_lo = slice * per;
    const int nkb = min(nkb_all, kb_lo + per);
    const int k_end = min(a.K, nkb * BK);       // loads at or beyond k_end return zeros

    // running position of this thread's vector in K: element index kv and, for tapped walks, (r, s, ci)
    int kv = kb_lo * BK + vcol * VEC;
    int kr = 0, ksx = 0, kci = kv;
    if constexpr (TAPS) {
        const int tap = div_by(kv, a.div_cin);
        kci = kv - tap * a.Cin;
        kr = div_by(tap, a.div_kw);
        ksx = tap - kr * a.kw;
    }

    // gather variant, short K: decode k -> (byte offset inside the window, tap row, tap col) once per workgroup
    constexpr int KTAB = LOAD == LOAD_GATHER ? 256 : 1;
    __shared__ int ktab_delta[KTAB], ktab_rq[KTAB];
    const bool use_ktab = LOAD == LOAD_GATHER && a.K <= KTAB;
    if constexpr (LOAD == LOAD_GATHER) {
        if (use_ktab) {
            for (int k = tid; k < a.K; k += THREADS) {
                const int tap = k / a.Cin, ci = k - tap * a.Cin;
                const int r = tap / a.kw, q = tap - r * a.kw;
                ktab_delta[k] = (int)((((int64_t)r * a.W + q) * a.x_pix + ci) * ESZ);
                ktab_rq[k] = (r << 8) | q;
            }
            __syncthreads();
        }
    }

    uint4 ra[2][AV], rb[2][BREG];
    // LOAD_AFFINE: scale and shift of this thread's channels of the block in flight, and the block's first channel
    constexpr bool PRE = LOAD == LOAD_AFFINE;
    constexpr int PV = PRE ? 2 * (VEC / 4) : 1;
    uint4 rp[2][PV];
    int rkv[2] = {0, 0};
    const bool pre_store = PRE && n0 == 0;      // the tile column that covers output channel 0 writes the affine tensor

    // loads the next K block of this thread (blocks are requested in ascending order, one call per block)
    auto load_global = [&](uint4 *pa, uint4 *pb, uint4 *pp, int &pkv) {
        if constexpr (LOAD == LOAD_GATHER) {
            // element-wise gather: any Cin, any alignment (stem convolutions, ragged K)
            T ea[AV][VEC], eb[BV][VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const int k = kv + e;
                const bool k_ok = k < k_end;
                int r, q;
                unsigned delta;
                if (use_ktab) {                 // short K (stem convolutions): k -> (offset, taps) from the LDS table
                    const int kc = k < KTAB ? k : KTAB - 1;
                    delta = (unsigned)ktab_delta[kc];
                    r = ktab_rq[kc] >> 8;
                    q = ktab_rq[kc] & 255;
                } else {
                    const int tap = k / a.Cin, ci = k - tap * a.Cin;
                    r = (tap / a.kw) & 31;
                    q = (tap - (tap / a.kw) * a.kw) & 31;
                    delta = (unsigned)((((int64_t)r * a.W + q) * a.x_pix + ci) * ESZ);
                }
#pragma unroll
                for (int i = 0; i < AV; ++i) {
                    const bool ok = k_ok && ((a_hm[i] >> r) & (a_wm[i] >> q) & 1u);
                    ea[i][e] = buf_load1<T>(xr, ok ? a_off[i] + delta : OOB);
                }
#pragma unroll
                for (int i = 0; i < BV; ++i) eb[i][e] = buf_load1<T>(wr, (k_ok && b_ok[i]) ? b_off[i] + (unsigned)(k * ESZ) : OOB);
            }
#pragma unroll
            for (int i = 0; i < AV; ++i) pa[i] = *(const uint4 *)ea[i];
#pragma unroll
            for (int i = 0; i < BV; ++i) pb[i] = *(const uint4 *)eb[i];
        } else {
            const bool k_ok = kv < k_end;
            if constexpr (TAPS) {
                const unsigned delta = (unsigned)((((int64_t)kr * a.W + ksx) * a.x_pix + kci) * ESZ);
                const unsigned tp = k_ok ? (unsigned)(kr * a.kw + ksx) : 31u;      // bit 31 is never set
#pragma unroll
                for (int i = 0; i < AV; ++i) pa[i] = buf_load16(xr, ((a_hm[i] >> tp) & 1u) ? a_off[i] + delta : OOB);
            } else {
                const unsigned delta = (unsigned)(kv * ESZ);
#pragma unroll
                for (int i = 0; i < AV; ++i) pa[i] = buf_load16(xr, (k_ok && a_hm[i]) ? a_off[i] + delta : OOB);
            }
            if constexpr (LOAD != LOAD_BT) {
                const unsigned delta = (unsigned)(kv * ESZ);
#pragma unroll
                for (int i = 0; i < BV; ++i) pb[i] = buf_load16(wr, (k_ok && b_ok[i]) ? b_off[i] + delta : OOB);
            } else {
                // B stored [k][n]: vectors run along n
                const int kb0 = kv - vcol * VEC;
#pragma unroll
                for (int i = 0; i < BTV; ++i) {
                    const int idx = tid + i * THREADS;
                    const int kk = idx / NV, nv = idx - kk * NV;
                    const int k = kb0 + kk, n = n0 + nv * VEC;
                    const bool ok = idx < BK * NV && k < k_end && n < a.n_hi;
                    pb[i] = buf_load16(wr, ok ? (unsigned)(((int64_t)k * a.w_row + n) * ESZ) : OOB);
                }
            }
        }
        if constexpr (PRE) {                    // beyond K both read zero, so the transformed element is act(0) = 0
            const __amdgpu_buffer_rsrc_t psr = make_rsrc(a.pre_scale, (int64_t)a.Cin * 4), phr = make_rsrc(a.pre_shift, (int64_t)a.Cin * 4);
            const bool k_ok = kv < k_end;
#pragma unroll
            for (int q = 0; q < VEC / 4; ++q) {
                pp[q] = buf_load16(psr, k_ok ? (unsigned)((kv + 4 * q) * 4) : OOB);
                pp[VEC / 4 + q] = buf_load16(phr, k_ok ? (unsigned)((kv + 4 * q) * 4) : OOB);
            }
            pkv = kv;
        }
        // advance to the next block
        kv += BK;
        if constexpr (TAPS) {
            kci += BK;
            if (a.Cin >= BK) {                  // at most one tap boundary per block: select-only update
                const bool w1 = kci >= a.Cin;
                kci -= w1 ? a.Cin : 0;
                ksx += w1 ? 1 : 0;
                const bool w2 = ksx == a.kw;
                ksx = w2 ? 0 : ksx;
                kr += w2 ? 1 : 0;
            } else {
                const int tap = div_by(kv, a.div_cin);
                kci = kv - tap * a.Cin;
                kr = div_by(tap, a.div_kw);
                ksx = tap - kr * a.kw;
            }
        }
    };

    auto store_lds = [&](int buf, const uint4 *pa, const uint4 *pb, const uint4 *pp, int pkv) {
        float sc[VEC], sh[VEC];
        if constexpr (PRE) {
#pragma unroll
            for (int q = 0; q < VEC / 4; ++q) {
                sc[4 * q] = __uint_as_float(pp[q].x); sc[4 * q + 1] = __uint_as_float(pp[q].y);
                sc[4 * q + 2] = __uint_as_float(pp[q].z); sc[4 * q + 3] = __uint_as_float(pp[q].w);
                sh[4 * q] = __uint_as_float(pp[VEC / 4 + q].x); sh[4 * q + 1] = __uint_as_float(pp[VEC / 4 + q].y);
                sh[4 * q + 2] = __uint_as_float(pp[VEC / 4 + q].z); sh[4 * q + 3] = __uint_as_float(pp[VEC / 4 + q].w);
            }
        }
#pragma unroll
        for (int i = 0; i < AV; ++i) {
            const int row = vrow + i * RPP;
            uint4 va = pa[i];
            if constexpr (PRE) {                // the stand-alone operator's arithmetic: one FMA, the activation, one rounding
                float v[VEC];
                if constexpr (DT == DT_BF16) {
                    const unsigned x4[4] = {va.x, va.y, va.z, va.w};
#pragma unroll
                    for (int q = 0; q < 4; ++q) { v[2 * q] = __uint_as_float(x4[q] << 16); v[2 * q + 1] = __uint_as_float(x4[q] & 0xFFFF0000u); }
                } else {
                    v[0] = __uint_as_float(va.x); v[1] = __uint_as_float(va.y); v[2] = __uint_as_float(va.z); v[3] = __uint_as_float(va.w);
                }
#pragma unroll
                for (int q = 0; q < VEC; ++q) {
                    const float t = __fmaf_rn(v[q], sc[q], sh[q]);
                    v[q] = a.pre_act == ACT_RELU ? __builtin_fmaxf(t, 0.f) : a.pre_act == ACT_RELU6 ? __builtin_amdgcn_fmed3f(t, 0.f, 6.f) : t;
                }
                if constexpr (DT == DT_BF16) {
                    va.x = (unsigned)to_bf16(v[0]) | ((unsigned)to_bf16(v[1]) << 16); va.y = (unsigned)to_bf16(v[2]) | ((unsigned)to_bf16(v[3]) << 16);
                    va.z = (unsigned)to_bf16(v[4]) | ((unsigned)to_bf16(v[5]) << 16); va.w = (unsigned)to_bf16(v[6]) | ((unsigned)to_bf16(v[7]) << 16);
                } else {
                    va = make_uint4(__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3]));
                }
                if (pre_store && a_hm[i] && pkv < k_end && (BM % RPP == 0 || row < BM))
                    *(uint4 *)((T *)a.pre_y + (int64_t)(m0 + row) * a.Cin + pkv) = va;
            }
            if (BM % RPP == 0 || row < BM) *(uint4 *)(As + (buf * BM + row) * ROWB + vcol * 16) = va;
        }
        if constexpr (LOAD != LOAD_BT) {
#pragma unroll
            for (int i = 0; i < BV; ++i) {
                const int row = vrow + i * RPP;
                if (BN % RPP == 0 || row < BN) *(uint4 *)(Bs + (buf * BN + row) * ROWB + vcol * 16) = pb[i];
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

    // Pipeline: LDS buffer p holds block kb, register set p^1 holds block kb+1 (in flight), and the loads
    // of block kb+2 are issued into register set p before the MFMAs of block kb start.  Loads and LDS
    // stores in the loop body are unconditional (blocks past the end of the slice read as zeros and land in
    // a buffer nobody reads), which keeps the body branch-free and the outstanding-load counts exact.
    load_global(ra[0], rb[0], rp[0], rkv[0]);
    store_lds(0, ra[0], rb[0], rp[0], rkv[0]);
    load_global(ra[1], rb[1], rp[1], rkv[1]);
    __syncthreads();
    int kb = kb_lo;
    for (; kb + 1 < nkb; kb += 2) {             // whole pairs of blocks; a single loop exit keeps one accumulator set
        load_global(ra[0], rb[0], rp[0], rkv[0]);
        compute(0);
        store_lds(1, ra[1], rb[1], rp[1], rkv[1]);
        __syncthreads();
        load_global(ra[1], rb[1], rp[1], rkv[1]);
        compute(1);
        store_lds(0, ra[0], rb[0], rp[0], rkv[0]);
        __syncthreads();
    }
    if (kb < nkb) compute(0);                   // odd block count: the last block already sits in LDS buffer 0
    __syncthreads();                            // the epilogue reuses the tile buffers

    igemm_epilogue<DT, BM, BN, WM, WN>(a, acc, (float *)smem + wave * (32 * 36), m0, n0, wm, wn, lane, slice, y_off);
}

// ------------------------------------------------------------------------------------------------
// The same product with the global -> LDS leg done by the memory pipeline itself ("buffer_load ... lds", 16 bytes per
// lane on gfx950): tiles go straight from L2 / HBM into LDS without passing through registers, so many K blocks can be
// in flight at once (NS stages of LDS) at no register cost.  What bounds the register-staged kernel above is the
// latency of its single block of prefetch, not a throughput; here block kb + NS - 1 is requested before block kb is
// consumed.
//
// Layout.  One such load makes a wave write 64 x 16 bytes back to back, so tile rows are unpadded (KV x 16 bytes) and
// consecutive lanes fill consecutive 16-byte slots: thread t owns slot t of every pass of 256 slots (RPP = 256 / KV
// tile rows per pass).  Bank conflicts of the fragment reads are avoided by an XOR swizzle instead of padding: the
// 16-byte chunk with logical index q of tile row r sits in slot q ^ swz(r), swz(r) = (r / (256 / ROWB)) % KV, which the
// loading lane applies on the global side (it fetches the logical chunk that belongs into its slot).
//
// Order of additions per output element is the one of igemm_kernel (ascending 32-byte k groups, zero fill beyond the
// K range; a stage that lies wholly beyond K multiplies zeros), so both kernels produce the same bits.
//
// Synchronisation: the loads are counted by vmcnt.  At the end of step kb the wave waits until only the loads of the
// NS - 2 youngest blocks are outstanding (block kb + 1 has landed), and for its own fragment reads, then meets the
// others at a bare s_barrier.  The stages are separate __shared__ arrays so that the compiler can see that a load
// into one stage does not alias the reads of another (with one array it waits for vmcnt(0) before every read).
#define GACER_LDS(p) ((__attribute__((address_space(3))) void *)(p))

template <int DT, int BM, int BN, int WM, int WN, int KV, int NS, bool TAPS>
__global__ __launch_bounds__(THREADS)
__attribute__((amdgpu_waves_per_eu(2 * NS * (BM + BN) * KV * 16 <= 160 * 1024 ? 2 : 1)))      // two workgroups per unit where LDS allows
void igemm_dma_kernel(GemmArgs a)
{
    typedef typename El<DT>::T T;
    constexpr int VEC = El<DT>::VEC;
    constexpr int ESZ = (int)sizeof(T);
    constexpr int BK = KV * VEC;
    constexpr int ROWB = KV * 16;               // unpadded tile row
    constexpr int RPP = THREADS / KV;           // tile rows covered by one pass of all threads
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    constexpr int AV = BM / RPP, BV = BN / RPP; // loads per thread and block
    constexpr int STAGE = (BM + BN) * ROWB;
    constexpr int R256 = 256 / ROWB;            // tile rows per 256 bytes of LDS (one sweep over the 64 banks)
    constexpr int PATCH = 32 * 36 * 4;          // bytes of one wave's epilogue patch
    constexpr bool OWN_PATCH = STAGE < PATCH * ((4 + NS - 1) / NS);
    static_assert(WM * WN == 4 && TM >= 1 && TN >= 1 && BM % RPP == 0 && BN % RPP == 0 && NS >= 3 && NS <= 8 && (KV == 4 || KV == 8), "tile shape");
    static_assert((NS - 2) * (AV + BV) < 64, "outstanding loads exceed the counter");

    __shared__ __align__(1024) unsigned char st0[STAGE];
    __shared__ __align__(1024) unsigned char st1[STAGE];
    __shared__ __align__(1024) unsigned char st2[STAGE];
    __shared__ __align__(1024) unsigned char st3[NS > 3 ? STAGE : 16];
    __shared__ __align__(1024) unsigned char st4[NS > 4 ? STAGE : 16];
    __shared__ __align__(1024) unsigned char st5[NS > 5 ? STAGE : 16];
    __shared__ __align__(1024) unsigned char st6[NS > 6 ? STAGE : 16];
    __shared__ __align__(1024) unsigned char st7[NS > 7 ? STAGE : 16];
    // the stages are separate arrays and always named by a compile-time index, so that the compiler can tell a stage
    // being filled from the one being read (it would otherwise wait for every outstanding load before each LDS read)
    auto stage_at = [&](int i) -> unsigned char * {
        return i == 0 ? st0 : i == 1 ? st1 : i == 2 ? st2 : i == 3 ? st3 : i == 4 ? st4 : i == 5 ? st5 : i == 6 ? st6 : st7;
    };
    __shared__ __align__(16) unsigned char own_patch[OWN_PATCH ? 4 * PATCH : 16];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int tile = xcd_contiguous((int)blockIdx.x, (int)gridDim.x);
    const int by_m = div_by(tile, a.div_tiles_m), by_n = div_by(tile, a.div_tiles_n);
    const int tile_m = __builtin_amdgcn_readfirstlane(a.n_major ? tile - by_m * a.tiles_m : by_n);
    const int tile_n = __builtin_amdgcn_readfirstlane(a.n_major ? by_m : tile - by_n * a.tiles_n);
    const int m0 = a.m_lo + tile_m * BM, n0 = a.n_lo + tile_n * BN;

    const int z = blockIdx.z;
    const int zq = __builtin_amdgcn_readfirstlane(div_by(z, a.div_zh));
    const int zb = a.z_lo + zq, zh = z - zq * a.zh;
    const int64_t x_zoff = zb * a.x_zb + zh * a.x_zh, w_zoff = zb * a.w_zb + zh * a.w_zh;
    const __amdgpu_buffer_rsrc_t xr = make_rsrc((const T *)a.x + x_zoff, a.x_bytes - x_zoff * ESZ);
    const __amdgpu_buffer_rsrc_t wr = make_rsrc((const T *)a.w + w_zoff, a.w_bytes - w_zoff * ESZ);
    const int64_t y_off = zb * a.y_zb + zh * a.y_zh;

    const int HoWo = a.Ho * a.Wo;
    const int vrow = tid / KV;                                  // tile row of this thread's slot in pass 0
    const int lcol = (tid % KV) ^ ((vrow / R256) % KV);         // logical chunk that belongs into the slot

    // per-thread A rows: byte offset of the window origin (or OOB) and one validity bit per tap
    unsigned a_off[AV], a_hm[AV];
#pragma unroll
    for (int i = 0; i < AV; ++i) {
        const int m = m0 + vrow + i * RPP;
        const bool ok = m < a.m_hi;
        const int mm = ok ? m : a.m_lo;
        const int img = div_by(mm, a.div_howo), rem = mm - img * HoWo;
        const int oh = div_by(rem, a.div_wo), ow = rem - oh * a.Wo;
        const int ih0 = oh * a.stride - a.pad, iw0 = ow * a.stride - a.pad;
        const int64_t e0 = (int64_t)img * a.x_img + ((int64_t)ih0 * a.W + iw0) * a.x_pix;   // may be negative at the border
        a_off[i] = ok ? (unsigned)(int)(e0 * ESZ) : OOB;
        a_hm[i] = ok ? tap_mask(ih0, iw0, a.H, a.W, a.kh, a.kw) : 0u;
    }
    unsigned b_off[BV];
#pragma unroll
    for (int i = 0; i < BV; ++i) {
        const int n = n0 + vrow + i * RPP;
        b_off[i] = n < a.n_hi ? (unsigned)((int64_t)n * a.w_row * ESZ) : OOB;
    }

    // K range of this slice, in blocks of BK (kb_per_slice counts 64-byte blocks)
    const int nkb_all = (a.K + BK - 1) / BK;
    const int per = a.kb_per_slice / (KV / 4);
    const int slice = blockIdx.y;
    const int kb_lo = slice * per;
    const int nkb = min(nkb_all, kb_lo + per);
    const int k_end = min(a.K, nkb * BK);       // loads at or beyond k_end return zeros

    int kv = kb_lo * BK + lcol * VEC;
    int kr = 0, ksx = 0, kci = kv;
    if constexpr (TAPS) {
        const int tap = div_by(kv, a.div_cin);
        kci = kv - tap * a.Cin;
        kr = div_by(tap, a.div_kw);
        ksx = tap - kr * a.kw;
    }

    // Requests for the next K block (one block per step, ascending).  A block is AV + BV loads per thread; they are issued
    // one at a time (request_part) so that a step can spread them between its MFMA groups: the unit that moves global
    // data into LDS takes the loads of all four waves in turn, and a wave that queues several at once is held there
    // while its matrix core runs dry.
    const int wave_slot = wave * 1024;
    bool rq_ok = false;
    unsigned rq_da = 0, rq_db = 0, rq_tap = 31u;
    auto request_begin = [&]() {
        rq_ok = kv < k_end;
        rq_db = (unsigned)(kv * ESZ);
        if constexpr (TAPS) {
            rq_da = (unsigned)((((int64_t)kr * a.W + ksx) * a.x_pix + kci) * ESZ);
            rq_tap = rq_ok ? (unsigned)(kr * a.kw + ksx) : 31u;                 // bit 31 is never set
        } else {
            rq_da = rq_db;
        }
    };
    auto request_part = [&](unsigned char *stage, int p) {                      // p in [0, AV + BV), a compile-time constant
        if (p < AV) {
            const int i = p;
            const bool ok = TAPS ? (((a_hm[i] >> rq_tap) & 1u) != 0) : (rq_ok && a_hm[i]);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xr, GACER_LDS(stage + i * RPP * ROWB + wave_slot), 16,
                                                     (int)(ok ? a_off[i] + rq_da : OOB), 0, 0, 0);
        } else {
            const int i = p - AV;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(wr, GACER_LDS(stage + (BM + i * RPP) * ROWB + wave_slot), 16,
                                                     (int)((rq_ok && b_off[i] != OOB) ? b_off[i] + rq_db : OOB), 0, 0, 0);
        }
    };
    auto request_end = [&]() {
        kv += BK;
        if constexpr (TAPS) {
            kci += BK;
            if (a.Cin >= BK) {                  // at most one tap boundary per block: select-only update
                const bool w1 = kci >= a.Cin;
                kci -= w1 ? a.Cin : 0;
                ksx += w1 ? 1 : 0;
                const bool w2 = ksx == a.kw;
                ksx = w2 ? 0 : ksx;
                kr += w2 ? 1 : 0;
            } else {
                const int tap = div_by(kv, a.div_cin);
                kci = kv - tap * a.Cin;
                kr = div_by(tap, a.div_kw);
                ksx = tap - kr * a.kw;
            }
        }
    };
    auto request = [&](unsigned char *stage) {                                  // a whole block at once (pipeline fill)
        request_begin();
#pragma unroll
        for (int p = 0; p < AV + BV; ++p) request_part(stage, p);
        request_end();
    };

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    const int lrow = lane & 31, lhalf = lane >> 5;
    // fragment reads: tile row lrow (+ a multiple of 32, which leaves the swizzle unchanged), logical chunk 2 g + lhalf
    const int frag_lo = (lhalf ^ ((lrow / R256) % KV)) * 16;
    const int a_row0 = (wm * (BM / WM) + lrow) * ROWB, b_row0 = (BM + wn * (BN / WN) + lrow) * ROWB;
    constexpr int G = KV / 2;                   // k groups (32 bytes of k) per block; group g lives in register set g & 1
    uint4 fa[2][TM], fb[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[1][i] = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[1][j] = make_uint4(0u, 0u, 0u, 0u);
    auto fragments = [&](const unsigned char *stage, int g, int set) {
        const int col = frag_lo ^ (g * 32);
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[set][i] = *(const uint4 *)(stage + a_row0 + i * 32 * ROWB + col);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[set][j] = *(const uint4 *)(stage + b_row0 + j * 32 * ROWB + col);
    };
    auto mfmas = [&](int set) {
        if constexpr (DT == DT_BF16) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[set][i]),
                                                                        __builtin_bit_cast(bf16x8, fb[set][j]), acc[i][j], 0, 0, 0);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const uint4 &va = fa[set][i], &vb = fb[set][j];
                        const float av = __uint_as_float(e == 0 ? va.x : e == 1 ? va.y : e == 2 ? va.z : va.w);
                        const float bv = __uint_as_float(e == 0 ? vb.x : e == 1 ? vb.y : e == 2 ? vb.z : vb.w);
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[i][j], 0, 0, 0);
                    }
        }
    };

    // vmcnt(N) & lgkmcnt(0): the loads of all but the NS - 2 youngest blocks have landed, own LDS reads are done
    constexpr int PENDING = (NS - 2) * (AV + BV);
    constexpr int WAIT_NEXT = (PENDING & 15) | (7 << 4) | ((PENDING >> 4) << 14);
    constexpr int WAIT_ALL = (7 << 4);
    auto meet = [&](int imm_is_all) {
        if (imm_is_all) __builtin_amdgcn_s_waitcnt(WAIT_ALL); else __builtin_amdgcn_s_waitcnt(WAIT_NEXT);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    // One step consumes block kb from `cur` and requests block kb + NS - 1 into the stage that block kb - 1 has left.
    // The step is rotated by one k group: the fragments of the last group of a block are in registers (set 1) when the
    // barrier is passed, and its MFMAs run first in the next step, covering the LDS latency of that step's first
    // fragments.  Slot 0 of a step is therefore the previous block's last group (before the first block: zeros, which
    // leave the accumulators at zero), slots 1 .. G - 1 are groups 0 .. G - 2 of this block.  Each slot issues the
    // fragment reads of the group after it and its share of the block's global requests, then its MFMAs; the
    // scheduling barriers keep that order in the generated code.  The chain of every accumulator still walks k upwards.
    constexpr int SCHED_ALU_MAY_CROSS = 0x2 | 0x4;       // vector and scalar ALU may move across; memory operations and MFMAs stay put
    auto step = [&](const unsigned char *cur, unsigned char *into) {
        request_begin();
#pragma unroll
        for (int slot = 0; slot < G; ++slot) {
            fragments(cur, slot, slot & 1);
#pragma unroll
            for (int p = slot * (AV + BV) / G; p < (slot + 1) * (AV + BV) / G; ++p) request_part(into, p);
            if (slot == G - 1) request_end();   // address arithmetic for the next block: free to mix with the MFMAs below
            __builtin_amdgcn_sched_barrier(SCHED_ALU_MAY_CROSS);
            mfmas((slot & 1) ^ 1);
            __builtin_amdgcn_sched_barrier(SCHED_ALU_MAY_CROSS);
        }
        meet(0);
    };

#pragma unroll
    for (int i = 0; i < NS - 1; ++i) request(stage_at(i));
    meet(0);                                    // block kb_lo has landed
    const int n_blocks = nkb - kb_lo;
    int done = 0;
    for (; done + NS <= n_blocks; done += NS) { // whole rounds over the stages; a single loop exit keeps one accumulator set
#pragma unroll
        for (int i = 0; i < NS; ++i) step(stage_at(i), stage_at((i + NS - 1) % NS));
    }
    const int rest = n_blocks - done;
#pragma unroll
    for (int i = 0; i < NS - 1; ++i)
        if (rest > i) step(stage_at(i), stage_at((i + NS - 1) % NS));
    mfmas(1);                                   // last group of the last block
    meet(1);                                    // trailing requests (all beyond K: zeros) have landed; the epilogue reuses the stages

    float *patch;
    if constexpr (OWN_PATCH) {
        patch = (float *)(own_patch + wave * PATCH);
    } else {
        const int which = wave % NS;
        unsigned char *base = stage_at(which);
        patch = (float *)(base + (wave / NS) * PATCH);
    }
    igemm_epilogue<DT, BM, BN, WM, WN>(a, acc, patch, m0, n0, wm, wn, lane, slice, y_off);
}

// ------------------------------------------------------------------------------------------------
// Row-streaming variant for pointwise (1x1, unpadded) convolutions and plain GEMMs with a short K: these
// are bound by HBM traffic, not by the matrix cores.  A wavefront owns 32 complete output rows: it reads
// its A fragments straight from global memory in MFMA operand layout (no LDS round trip, no workgroup
// barrier in the loop), takes the B fragments of all 32*TN output channels from an LDS copy made once per
// workgroup, and turns the accumulators through a private LDS patch so that residual loads and output
// stores are contiguous 16-byte vectors along the channel axis, written back to back by the same wave.
// Every accumulator is the same MFMA chain over ascending 32-byte k groups as in igemm_kernel, so both
// kernels produce the same bits.
template <int DT, int TN, int G>
__global__ __launch_bounds__(THREADS) void rowgemm_kernel(GemmArgs a)
{
    typedef typename El<DT>::T T;
    constexpr int VEC = El<DT>::VEC;
    constexpr int ESZ = (int)sizeof(T);
    constexpr int EV = DT == DT_BF16 ? 8 : 4;
    constexpr int HALF = 64;                          // staged columns per pass
    constexpr int SROW = HALF + 4;                    // floats per staged row
    extern __shared__ __align__(16) unsigned char dyn_smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lrow = lane & 31, lhalf = lane >> 5;
    const int kg = (a.K * ESZ + 31) / 32;             // 32-byte k groups
    const int kg4 = (kg + 3) & ~3;                // LDS rows hold whole groups of four
    const int kgr = (kg + G - 1) / G * G;          // groups walked: G at a time (G = 1 for very short K)
    const int rowb = kg4 * 32 + 16;                   // LDS bytes per B row
    unsigned char *Bs = dyn_smem;
    float *stage = (float *)(dyn_smem + 32 * TN * rowb) + wave * (32 * SROW);

    const int n0 = a.n_lo + (int)blockIdx.y * (32 * TN);
    const int m0 = a.m_lo + (int)blockIdx.x * 128 + wave * 32;
    const __amdgpu_buffer_rsrc_t xr = make_rsrc(a.x, a.x_bytes);
    const __amdgpu_buffer_rsrc_t wr = make_rsrc(a.w, a.w_bytes);

    // B rows of this channel group -> LDS (zero beyond K and beyond the launched channel range)
    for (int r = tid >> 3; r < 32 * TN; r += THREADS / 8)
        for (int v = tid & 7; v < kg4 * 2; v += 8) {
            const int n = n0 + r, k = v * VEC;
            const bool ok = n < a.n_hi && k < a.K;
            *(uint4 *)(Bs + r * rowb + v * 16) = buf_load16(wr, ok ? (unsigned)(((int64_t)n * a.w_row + k) * ESZ) : OOB);
        }
    // this lane's A row
    unsigned a_off;
    {
        const int m = m0 + lrow;
        const bool ok = m < a.m_hi;
        const int mm = ok ? m : a.m_lo;
        int64_t e0;
        if (a.stride == 1 && a.x_img == (int64_t)a.Ho * a.Wo * a.x_pix) {      // dense rows: no index arithmetic
            e0 = (int64_t)mm * a.x_pix;
        } else {
            const int HoWo = a.Ho * a.Wo;
            const int img = div_by(mm, a.div_howo), rem = mm - img * HoWo;
            const int oh = div_by(rem, a.div_wo), ow = rem - oh * a.Wo;
            e0 = (int64_t)img * a.x_img + ((int64_t)oh * a.stride * a.W + ow * a.stride) * a.x_pix;
        }
        a_off = ok ? (unsigned)(e0 * ESZ) : OOB;
    }
    const unsigned k_bytes = (unsigned)(a.K * ESZ);
    auto load4 = [&](uint4 *f, int g0) {
#pragma unroll
        for (int q = 0; q < G; ++q) {
            const unsigned kb = (unsigned)((g0 + q) * 32 + lhalf * 16);
            f[q] = buf_load16(xr, (a_off != OOB && kb < k_bytes) ? a_off + kb : OOB);
        }
    };

    f32x16 acc[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;

    auto compute4 = [&](const uint4 *f, int g0) {
#pragma unroll
        for (int q = 0; q < G; ++q) {
            uint4 fb[TN];
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[j] = *(const uint4 *)(Bs + (j * 32 + lrow) * rowb + (g0 + q) * 32 + lhalf * 16);
            if constexpr (DT == DT_BF16) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, f[q]), __builtin_bit_cast(bf16x8, fb[j]),
                                                                     acc[j], 0, 0, 0);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int j = 0; j < TN; ++j) {
                        const float av = __uint_as_float(e == 0 ? f[q].x : e == 1 ? f[q].y : e == 2 ? f[q].z : f[q].w);
                        const float bv = __uint_as_float(e == 0 ? fb[j].x : e == 1 ? fb[j].y : e == 2 ? fb[j].z : fb[j].w);
                        acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[j], 0, 0, 0);
                    }
            }
        }
    };

    uint4 fa[2][G];
    load4(fa[0], 0);
    __syncthreads();
    int g0 = 0;
    for (; g0 + G < kgr; g0 += 2 * G) {
        load4(fa[1], g0 + G);
        compute4(fa[0], g0);
        load4(fa[0], g0 + 2 * G);
        compute4(fa[1], g0 + G);
    }
    if (g0 < kgr) compute4(fa[0], g0);

    // ---- epilogue: 64 channels at a time through the wave's LDS patch ----
    constexpr int CPR = HALF / EV;                    // 16-byte chunks per staged row
    constexpr int RPI = 64 / CPR;                     // rows per pass of the wave
    T *yg = (T *)a.y;
    const T *rg = (const T *)a.res;
    const bool vec_out = a.y_row % EV == 0 && a.n_lo % EV == 0 && (((uintptr_t)a.y) & 15) == 0 && (((uintptr_t)a.res) & 15) == 0 &&
                         (((uintptr_t)a.bias) & 15) == 0;
#pragma unroll
    for (int hf = 0; hf < (TN + 1) / 2; ++hf) {
        constexpr int ITER = 32 / RPI;
        const int width = (hf * 2 + 1 < TN) ? HALF : 32;
        const int col = (lane % CPR) * EV, n = n0 + hf * HALF + col;
        const bool n_ok = col < width && n < a.n_hi;
        const bool n_vec = n_ok && vec_out && n + EV <= a.n_hi;
        // bias and residual loads before the LDS turn (see igemm_kernel)
        float bv[EV];
        load_bias_vec<EV>(a.bias, n, n_vec, bv);
        uint4 rv[ITER];
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            const int m = m0 + it * RPI + lane / CPR;
            rv[it] = make_uint4(0u, 0u, 0u, 0u);
            if (rg && n_vec && m < a.m_hi) rv[it] = *(const uint4 *)(rg + (int64_t)m * a.y_row + n);
        }
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int j = hf * 2 + jj;
            if (j < TN) {
#pragma unroll
                for (int e = 0; e < 16; ++e) stage[((e >> 2) * 8 + lhalf * 4 + (e & 3)) * SROW + jj * 32 + lrow] = acc[j < TN ? j : 0][e];
            }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            const int row = it * RPI + lane / CPR;
            const int m = m0 + row;
            float v[EV];
#pragma unroll
            for (int q = 0; q < EV; q += 4) {
                const float4 t4 = *(const float4 *)(stage + row * SROW + col + q);
                v[q] = t4.x; v[q + 1] = t4.y; v[q + 2] = t4.z; v[q + 3] = t4.w;
            }
            if (!n_ok || m >= a.m_hi) continue;
            const int64_t o = (int64_t)m * a.y_row + n;
            if (n_vec) finish_vec<DT>(a, v, bv, rg != nullptr, rv[it], yg, o);
            else finish_scalar<DT>(a, v, rg, yg, o, n);
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// Second pass of a split-K operator: out = act(alpha * (s0 + s1 + ... ) + bias + res), slices added in
// ascending order.  One thread per FV consecutive output channels of the launched sub-range (FV = 4 when
// the range and the pointers allow 16-byte accesses), coalesced along n.
template <typename T, int FV>
__global__ __launch_bounds__(THREADS) void splitk_finish(GemmArgs a)
{
    const int Nl = a.n_hi - a.n_lo;
    const int64_t total = (int64_t)(a.m_hi - a.m_lo) * Nl;
    const int64_t idx = ((int64_t)blockIdx.x * THREADS + threadIdx.x) * FV;
    if (idx >= total) return;
    const int mr = div_by((int)idx, a.div_nl);          // idx < 2^31: the launched sub-range holds fewer elements
    const int m = a.m_lo + mr, n = a.n_lo + ((int)idx - mr * Nl);
    const int64_t o = (int64_t)m * a.y_row + n;
    // bias and residual are requested together with the slices: one global round trip for the whole kernel
    float bv[FV], rv[FV];
#pragma unroll
    for (int e = 0; e < FV; ++e) bv[e] = a.bias ? a.bias[n + e] : 0.f;
#pragma unroll
    for (int e = 0; e < FV; ++e) rv[e] = a.res ? load_in((const T *)a.res, o + e) : 0.f;
    float v[FV];
    if constexpr (FV == 4) {
        float4 p[16];                          // all slice loads are issued before the first add (ksplit <= 16)
#pragma unroll
        for (int q = 0; q < 16; ++q) p[q] = q < a.ksplit ? *(const float4 *)(a.ws + q * total + idx) : make_float4(0.f, 0.f, 0.f, 0.f);
        v[0] = p[0].x; v[1] = p[0].y; v[2] = p[0].z; v[3] = p[0].w;
#pragma unroll
        for (int q = 1; q < 16; ++q)
            if (q < a.ksplit) {
                v[0] = __fadd_rn(v[0], p[q].x); v[1] = __fadd_rn(v[1], p[q].y);
                v[2] = __fadd_rn(v[2], p[q].z); v[3] = __fadd_rn(v[3], p[q].w);
            }
    } else {
        float p[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) p[q] = q < a.ksplit ? a.ws[q * total + idx] : 0.f;
        v[0] = p[0];
#pragma unroll
        for (int q = 1; q < 16; ++q)
            if (q < a.ksplit) v[0] = __fadd_rn(v[0], p[q]);
    }
#pragma unroll
    for (int e = 0; e < FV; ++e) {
        float t = __fmaf_rn(v[e], a.alpha, bv[e]);
        if (a.res) t = __fadd_rn(t, rv[e]);
        v[e] = act_apply(t, a.act);
    }
    if constexpr (FV == 4 && sizeof(T) == 4) {
        *(float4 *)((float *)a.y + o) = make_float4(v[0], v[1], v[2], v[3]);
    } else if constexpr (FV == 4) {
        *(uint2 *)((unsigned short *)a.y + o) = make_uint2(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]));
    } else {
        store_out<T>((T *)a.y, o, v[0]);
    }
}

template <typename T>
static void launch_finish(const GemmArgs &a, hipStream_t s)
{
    const int Nl = a.n_hi - a.n_lo;
    const int64_t total = (int64_t)(a.m_hi - a.m_lo) * Nl;
    const bool v4 = Nl % 4 == 0 && a.n_lo % 4 == 0 && a.y_row % 4 == 0 && (((uintptr_t)a.ws) & 15) == 0 && (((uintptr_t)a.y) & 15) == 0;
    GemmArgs b = a;
    divisor(Nl, b.div_nl);
    if (v4)
        GACER_LAUNCH((splitk_finish<T, 4>), dim3((unsigned)((total / 4 + THREADS - 1) / THREADS)), dim3(THREADS), 0, s, b);
    else
        GACER_LAUNCH((splitk_finish<T, 1>), dim3((unsigned)((total + THREADS - 1) / THREADS)), dim3(THREADS), 0, s, b);
}

static void set_tiling(GemmArgs &b, int tiles_m, int tiles_n)
{
    b.tiles_m = tiles_m;
    b.tiles_n = tiles_n;
    divisor(tiles_m, b.div_tiles_m);
    divisor(tiles_n, b.div_tiles_n);
    divisor(b.zh, b.div_zh);
}
static void set_divisors(GemmArgs &b)
{
    divisor(b.Ho * b.Wo, b.div_howo);
    divisor(b.Wo, b.div_wo);
    divisor(b.Cin, b.div_cin);
    divisor(b.kw, b.div_kw);
}

// Tile numbering of a launch.  m-major numbering gives every XCD a band of output rows: A is fetched into one L2 only,
// B into every L2 that holds a band; n-major numbering is the mirror image.  Takes the order that moves fewer bytes
// into the L2s (late convolution layers have far more weights than activations, early ones the opposite).
static int tile_order(const GemmArgs &a, int tiles_m, int tiles_n, int esz)
{
    const double Ml = a.m_hi - a.m_lo, Nl = a.n_hi - a.n_lo;
    const double A = Ml * a.stride * a.stride * (double)(a.K / (a.kh * a.kw)) * esz;     // input pixels behind the output rows
    const double B = Nl * (double)a.K * esz;
    const double m_major = A + (tiles_m < 8 ? tiles_m : 8) * B, n_major = B + (tiles_n < 8 ? tiles_n : 8) * A;
    return n_major < m_major ? 1 : 0;
}

// ------------------------------------------------------------------------------------------------
template <int DT, int BM, int BN, int WM, int WN, int KV>
static LaunchInfo go(const GemmArgs &a, hipStream_t s, bool dry, bool vec_ok, int phase)
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
    static const std::string n_vec = "igemm_" + shape, n_bt = "igemm_bt_" + shape, n_gather = "igemm_gather_" + shape,
                             n_taps = "igemm_taps_" + shape, n_pre = "igemm_affine_" + shape;
    const bool taps = !(a.kh == 1 && a.kw == 1 && a.pad == 0);
    if (taps && a.kh * a.kw > 31) vec_ok = false;      // the tapped loader keeps one validity bit per tap in a 32-bit mask
    li.kernel = a.pre_scale ? n_pre.c_str() : a.b_trans ? n_bt.c_str() : (!vec_ok ? n_gather.c_str() : (taps ? n_taps.c_str() : n_vec.c_str()));
    li.phases = ks > 1 ? 2 : 1;
    if (phase == 2) li.kernel = "splitk_finish";
    if (dry || li.workgroups == 0) return li;
    dim3 grid(tiles_m * tiles_n, ks, z), block(THREADS);
    if (phase == 2) {
        if (ks > 1) launch_finish<T>(a, s);
        return li;
    }
    GemmArgs b = a;
    b.n_major = tile_order(a, tiles_m, tiles_n, (int)sizeof(T));
    set_divisors(b);
    set_tiling(b, tiles_m, tiles_n);
    if (a.pre_scale)
        GACER_LAUNCH((igemm_kernel<DT, BM, BN, WM, WN, KV, LOAD_AFFINE>), grid, block, 0, s, b);
    else if (a.b_trans)
        GACER_LAUNCH((igemm_kernel<DT, BM, BN, WM, WN, KV, LOAD_BT>), grid, block, 0, s, b);
    else if (!vec_ok)
        GACER_LAUNCH((igemm_kernel<DT, BM, BN, WM, WN, KV, LOAD_GATHER>), grid, block, 0, s, b);
    else if (taps)
        GACER_LAUNCH((igemm_kernel<DT, BM, BN, WM, WN, KV, LOAD_TAPS>), grid, block, 0, s, b);
    else
        GACER_LAUNCH((igemm_kernel<DT, BM, BN, WM, WN, KV, LOAD_VEC>), grid, block, 0, s, b);
    if (ks > 1 && phase == 0) launch_finish<T>(a, s);
    return li;
}

// launcher of igemm_dma_kernel (operands 16-byte aligned in every stride, B rows contiguous in k, at most 31 taps)
template <int DT, int BM, int BN, int WM, int WN, int KV, int NS>
static LaunchInfo go_dma(const GemmArgs &a, hipStream_t s, bool dry, bool vec_ok, int phase)
{
    typedef typename El<DT>::T T;
    constexpr int STAGE = (BM + BN) * KV * 16, PATCH = 32 * 36 * 4;
    constexpr bool OWN_PATCH = STAGE < PATCH * ((4 + NS - 1) / NS);
    const int tiles_m = (a.m_hi - a.m_lo + BM - 1) / BM, tiles_n = (a.n_hi - a.n_lo + BN - 1) / BN;
    const int z = a.zb * a.zh;
    const int ks = a.ksplit;
    LaunchInfo li;
    li.workgroups = tiles_m * tiles_n * z * ks;
    li.threads = THREADS;
    li.lds_bytes = NS * STAGE + (OWN_PATCH ? 4 * PATCH : 0);
    const int by_lds = (160 * 1024) / li.lds_bytes;
    li.wg_per_cu = by_lds < 8 ? by_lds : 8;
    static const std::string shape = std::string(DT == DT_BF16 ? "bf16_" : "f32_") + std::to_string(BM) + "x" + std::to_string(BN) +
                                     "x" + std::to_string(KV * El<DT>::VEC) + "s" + std::to_string(NS);
    static const std::string n_one = "igemm_dma_" + shape, n_taps = "igemm_dma_taps_" + shape;
    const bool taps = !(a.kh == 1 && a.kw == 1 && a.pad == 0);
    li.kernel = taps ? n_taps.c_str() : n_one.c_str();
    li.phases = ks > 1 ? 2 : 1;
    if (phase == 2) li.kernel = "splitk_finish";
    if (dry || li.workgroups == 0) return li;
    dim3 grid(tiles_m * tiles_n, ks, z), block(THREADS);
    if (phase == 2) {
        if (ks > 1) launch_finish<T>(a, s);
        return li;
    }
    GemmArgs b = a;
    b.n_major = tile_order(a, tiles_m, tiles_n, (int)sizeof(T));
    set_divisors(b);
    set_tiling(b, tiles_m, tiles_n);
    if (taps) GACER_LAUNCH((igemm_dma_kernel<DT, BM, BN, WM, WN, KV, NS, true>), grid, block, 0, s, b);
    else GACER_LAUNCH((igemm_dma_kernel<DT, BM, BN, WM, WN, KV, NS, false>), grid, block, 0, s, b);
    if (ks > 1 && phase == 0) launch_finish<T>(a, s);
    return li;
}

// rowgemm_kernel is taken when the operator is a single-tap, unpadded, unsplit bf16 product whose rows are at most
// 192 bytes of K (measured: beyond that, and for fp32 at any K, the tiled kernel is as fast or faster): properties
// of the operator, not of the launched sub-range, so every chunk of an operator takes the same path as its
// unsplit launch.
static bool rows_eligible(const GemmArgs &a, int esz, bool vec_ok)
{
    return vec_ok && !a.b_trans && a.ksplit == 1 && a.kh == 1 && a.kw == 1 && a.pad == 0 && a.zb * a.zh == 1 && a.z_lo == 0 &&
           esz == 2 && (int64_t)a.K * esz <= 192;
}
static int rows_lds(int tn, int K, int esz)
{
    const int kg4 = (((K * esz + 31) / 32) + 3) & ~3;
    return 32 * tn * (kg4 * 32 + 16) + 4 * 32 * 68 * 4;
}

template <int DT, int TN, int G>
static LaunchInfo go_rows_g(const GemmArgs &a, hipStream_t s, const LaunchInfo &li, int groups)
{
    GemmArgs b = a;
    set_divisors(b);
    GACER_LAUNCH((rowgemm_kernel<DT, TN, G>), dim3((a.m_hi - a.m_lo + 127) / 128, groups), dim3(THREADS), li.lds_bytes, s, b);
    return li;
}

template <int DT, int TN>
static LaunchInfo go_rows(const GemmArgs &a, hipStream_t s, bool dry, int groups)
{
    LaunchInfo li;
    const int M = a.m_hi - a.m_lo;
    li.workgroups = ((M + 127) / 128) * groups;
    li.threads = THREADS;
    li.lds_bytes = rows_lds(TN, a.K, (int)sizeof(typename El<DT>::T));
    const int by_lds = (160 * 1024) / li.lds_bytes;
    li.wg_per_cu = by_lds < 8 ? by_lds : 8;
    static const std::string name = std::string("rowgemm_") + (DT == DT_BF16 ? "bf16" : "f32") + "_x" + std::to_string(32 * TN);
    li.kernel = name.c_str();
    li.phases = 1;
    if (dry || li.workgroups == 0) return li;
    const int kg = (a.K * (int)sizeof(typename El<DT>::T) + 31) / 32;
    return kg < 4 ? go_rows_g<DT, TN, 1>(a, s, li, groups) : go_rows_g<DT, TN, 4>(a, s, li, groups);
}

template <int DT>
static LaunchInfo pick_rows(const GemmArgs &a, hipStream_t s, bool dry)
{
    const int esz = (int)sizeof(typename El<DT>::T);
    const int N = a.n_hi - a.n_lo, t32 = (N + 31) / 32;
    int tn_max = 6;
    while (tn_max > 1 && rows_lds(tn_max, a.K, esz) > 64 * 1024) --tn_max;
    int groups = (t32 + tn_max - 1) / tn_max;
    // few rows: spread the channels over more workgroups until every compute unit has one (A is then re-read from L2)
    const int wgs_m = (a.m_hi - a.m_lo + 127) / 128;
    while (groups < t32 && wgs_m * groups < 256) ++groups;
    const int tn = (t32 + groups - 1) / groups;
    groups = (t32 + tn - 1) / tn;
    switch (tn) {
    case 1: return go_rows<DT, 1>(a, s, dry, groups);
    case 2: return go_rows<DT, 2>(a, s, dry, groups);
    case 3: return go_rows<DT, 3>(a, s, dry, groups);
    case 4: return go_rows<DT, 4>(a, s, dry, groups);
    case 5: return go_rows<DT, 5>(a, s, dry, groups);
    default: return go_rows<DT, 6>(a, s, dry, groups);
    }
}

template <int DT>
static LaunchInfo pick(const GemmArgs &a, hipStream_t s, bool dry, int phase)
{
    constexpr int VEC = El<DT>::VEC;
    const bool vec_ok = (a.Cin % VEC == 0) && (a.x_pix % VEC == 0) && (a.x_img % VEC == 0) && (a.w_row % VEC == 0) &&
                        (a.x_zb % VEC == 0) && (a.x_zh % VEC == 0) && (a.w_zb % VEC == 0) && (a.w_zh % VEC == 0) &&
                        (((uintptr_t)a.x) % 16 == 0) && (((uintptr_t)a.w) % 16 == 0);
    if constexpr (DT == DT_BF16) {
        if (!a.pre_scale && rows_eligible(a, (int)sizeof(typename El<DT>::T), vec_ok)) return pick_rows<DT>(a, s, dry || phase == 2);
    }
    const int M = a.m_hi - a.m_lo, N = a.n_hi - a.n_lo;
    const int64_t z = (int64_t)a.zb * a.zh * (a.b_trans ? 1 : a.ksplit);
    // Tile choice is free (it never changes the bits): narrowest N padding first, then the cheapest shape.
    auto waste = [&](int bn) { return (double)((N + bn - 1) / bn * bn) / (double)N; };
    int bn = 128;
    if (waste(64) < waste(bn) - 1e-9) bn = 64;
    if (waste(32) < waste(bn) - 1e-9) bn = 32;
    auto wgs = [&](int bm, int bnn) { return (int64_t)((M + bm - 1) / bm) * ((N + bnn - 1) / bnn) * z; };
    // Cost of a tile shape: workgroups landing on the busiest compute unit x outputs per workgroup / relative
    // efficiency of the shape.  Measured: bf16 gains from the 128x128 tile (fewer LDS reads per MFMA), the two
    // smaller shapes are equal; fp32 MFMAs are slow enough that all shapes are equal and only the fill counts.
    // Fewer workgroups than compute units leaves units idle and hides no latency: penalised.
    constexpr double e_small = DT == DT_BF16 ? 0.8 : 1.0, e_mid = e_small;
    auto cost = [&](int bm, int bnn, double eff) {
        const int64_t w = wgs(bm, bnn);
        return (double)((w + 255) / 256) * bm * bnn / eff * (w < 256 ? 1.1 : 1.0);
    };
    int shape = 0;                               // 0: 64x64, 1: 128x64, 2: 128x128, 3: 128x32
    if (bn < 64) shape = 3;
    else {
        double best = cost(64, 64, e_small);
        if (cost(128, 64, e_mid) < best * 0.999) { best = cost(128, 64, e_mid); shape = 1; }
        if (bn == 128 && cost(128, 128, 1.0) < best * 0.999) shape = 2;
    }
    if (a.pre_scale) {                           // fused per-channel affine: the A tile passes through registers, so the register-staged kernel
        switch (shape) {                         // (the executor fuses only 16-byte aligned, vector-multiple operands)
        case 2: return go<DT, 128, 128, 2, 2, 8>(a, s, dry, true, phase);
        case 1: return go<DT, 128, 64, 2, 2, 8>(a, s, dry, true, phase);
        case 0: return go<DT, 64, 64, 2, 2, 8>(a, s, dry, true, phase);
        default: return go<DT, 128, 32, 4, 1, 8>(a, s, dry, true, phase);
        }
    }
    // Long K rows: the direct-to-LDS pipeline (igemm_dma_kernel) keeps several K blocks in flight and wins once the K
    // loop is long enough to amortise filling its stages (measured layer by layer: from about 1.5 KB of K per row).
    const bool taps = !(a.kh == 1 && a.kw == 1 && a.pad == 0);
    if (vec_ok && !a.b_trans && shape != 3 && (!taps || a.kh * a.kw <= 31) && (int64_t)a.K * (int64_t)sizeof(typename El<DT>::T) >= 1536) {
        const bool long_k = (int64_t)a.K * (int64_t)sizeof(typename El<DT>::T) >= 4096;
        if (shape == 2) {
            // 256x128 halves the L2 traffic of the A operand per flop again; it needs enough rows to still fill the chip
            if (DT == DT_BF16 && wgs(256, 128) >= 384) return go_dma<DT, 256, 128, 2, 2, 4, 3>(a, s, dry, vec_ok, phase);
            // one workgroup per compute unit anyway: whole 128-byte row segments (fewer, larger L2 requests)
            if (wgs(128, 128) <= 256) return go_dma<DT, 128, 128, 2, 2, 8, 3>(a, s, dry, vec_ok, phase);
            return go_dma<DT, 128, 128, 2, 2, 4, 4>(a, s, dry, vec_ok, phase);
        }
        if (shape == 1) return go_dma<DT, 128, 64, 2, 2, 8, 3>(a, s, dry, vec_ok, phase);
        if (long_k && DT == DT_BF16) return go_dma<DT, 64, 64, 2, 2, 8, 4>(a, s, dry, vec_ok, phase);   // measured: a fourth stage pays for bf16 only
        return go_dma<DT, 64, 64, 2, 2, 8, 3>(a, s, dry, vec_ok, phase);
    }
    if (a.b_trans || a.K <= 16 * VEC || !vec_ok) {   // short K, or the latency-bound gather loader (more waves per unit): 64-byte blocks
        switch (shape) {
        case 2: return go<DT, 128, 128, 2, 2, 4>(a, s, dry, vec_ok, phase);
        case 1: return go<DT, 128, 64, 2, 2, 4>(a, s, dry, vec_ok, phase);
        case 0: return go<DT, 64, 64, 2, 2, 4>(a, s, dry, vec_ok, phase);
        default: return go<DT, 128, 32, 4, 1, 4>(a, s, dry, vec_ok, phase);
        }
    }
    switch (shape) {
    case 2: return go<DT, 128, 128, 2, 2, 8>(a, s, dry, vec_ok, phase);
    case 1: return go<DT, 128, 64, 2, 2, 8>(a, s, dry, vec_ok, phase);
    case 0: return go<DT, 64, 64, 2, 2, 8>(a, s, dry, vec_ok, phase);
    default: return go<DT, 128, 32, 4, 1, 8>(a, s, dry, vec_ok, phase);
    }
}

LaunchInfo launch_igemm(const GemmArgs &a, hipStream_t s, bool dry, int phase)
{
    return a.dtype == DT_BF16 ? pick<DT_BF16>(a, s, dry, phase) : pick<DT_F32>(a, s, dry, phase);
}

}  // namespace gacer
