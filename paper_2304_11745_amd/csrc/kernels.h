// Internal launch interface between the executor and the gfx950 kernels.
// Every launcher enqueues exactly one kernel on `s` covering only the requested sub-range
// (a decomposed operator chunk, Eq. 5, is a real smaller launch).  Launchers validate nothing:
// the executor checks shapes when tenants are loaded and sub-ranges when a plan is set.
#pragma once
#include <hip/hip_runtime_api.h>
#include <stdint.h>

namespace gacer {

enum { DT_F32 = 0, DT_BF16 = 1 };
enum { ACT_NONE = 0, ACT_RELU = 1, ACT_RELU6 = 2, ACT_GELU = 3, ACT_HSWISH = 4, ACT_HSIGMOID = 5 };

// Implicit-GEMM view of conv / GEMM / attention products:  Y[m][n] = sum_k A[m][k] * B[n][k].
//   rows m  = output positions (image, oh, ow), cols n = output channels, k = (tap r, tap s, ci).
//   A is gathered from a channels-last tensor, B rows are contiguous in k (b_trans == 0) or
//   B is stored [k][n] (b_trans == 1, attention values).
// z = blockIdx.z walks `zb * zh` independent problems (attention: batch x heads) through the
// *_zb / *_zh element offsets.
struct GemmArgs {
    const void *x, *w;
    int64_t x_bytes, w_bytes;  // bytes from x / w to the end of their tensors (bounds of the buffer descriptors)
    const float *bias;
    const void *res;
    void *y;
    int dtype;
    int H, W, Cin;             // input extent per image and channels read per tap
    int Ho, Wo;                // output extent per image
    int kh, kw, stride, pad;
    int K;                     // kh*kw*Cin
    int64_t x_pix;             // elements between neighbouring input pixels
    int64_t x_img;             // elements between images
    int64_t w_row;             // elements between B rows (b_trans: between k rows)
    int64_t y_row;             // elements between output rows (also used for res)
    int m_lo, m_hi;            // output row sub-range
    int n_lo, n_hi;            // output channel sub-range
    int act;
    float alpha;               // scale applied to the accumulator before bias
    int b_trans;
    int zb, zh;
    int64_t x_zb, x_zh, w_zb, w_zh, y_zb, y_zh;
    int z_lo;                  // first zb index of the sub-range (zb counts problems launched)
    // Split-K: the K blocks are cut into `ksplit` slices of `kb_per_slice` 64-byte blocks.  Each slice is
    // accumulated by its own workgroup into `ws` ([slice][row][col] floats over the launched sub-range); a
    // second kernel adds the slices in order 0,1,2,... and applies the epilogue.  Both numbers are fixed per
    // operator from its unsplit shape, so every decomposition adds in the same order.
    int ksplit, kb_per_slice;
    float *ws;
    int n_major;               // set by the launcher: tiles are numbered n-major (1) or m-major (0), see tile_order()
    // set by the launcher: n / d for 0 <= n < 2^31 as (n * mul) >> (32 + shift), mul = 0 meaning d = 1; d = Ho*Wo, Wo, Cin, kw
    unsigned div_howo[2], div_wo[2], div_cin[2], div_kw[2];
    // set by the launcher of the tiled kernels: tiles along m and n of this launch, divisors for them and for zh
    int tiles_m, tiles_n;
    unsigned div_tiles_m[2], div_tiles_n[2], div_zh[2];
    unsigned div_nl[2];        // set by the launcher of the finishing pass: divisor for n_hi - n_lo
    // Per-channel affine + activation fused in front of a 1x1 product (pre_scale != null): x is the affine operator's INPUT
    // (same shape as its output, K = Cin channels) and A[m][k] = pre_act(x[m][k] * pre_scale[k] + pre_shift[k]), rounded to
    // the element type, is formed while the A tile is stored to LDS; the tiles that cover output channel 0 also write it to
    // pre_y ([rows][Cin]), so the affine operator's output tensor exists as if its own kernel had run.  pre_act is
    // ACT_NONE, ACT_RELU or ACT_RELU6 (zero stays zero, which the zero fill beyond K relies on).
    const float *pre_scale, *pre_shift;
    void *pre_y;
    int pre_act;
};

// Channels-last streaming operators.  Sub-range: images [n_lo,n_hi), channels [c_lo,c_hi).
struct StreamArgs {
    const void *x, *x2, *res, *w;
    const float *bias, *scale, *shift;
    void *y;
    int dtype;
    int N, H, W, C, Ho, Wo;
    int k, stride, pad;
    int act;
    float eps;
    int n_lo, n_hi, c_lo, c_hi;
    int64_t rows_per_item;     // row operators: rows (positions) per batch item
    const void *gate;          // eltwise: per-(image, channel) factor [N][C] in the tensor dtype, or null
    int c_split;               // concat: channels of x (the first input); the rest of C come from x2
    int pool_avg;              // pooling: 0 = window maximum, 1 = unpadded window mean
    int64_t x_pitch, y_pitch;  // eltwise (x, y) and pooling (y): elements between neighbouring positions (C unless the tensor is a channel window)
    // set by the launcher (see GemmArgs): divisors for the channel vectors per position, the positions (or position
    // tiles) per output row, and the output rows per image of this launch
    unsigned div_cv[2], div_w[2], div_h[2];
};

// Per-kernel timing (measurement aid): while `launch_timer` points at an event pair on the calling thread, every
// launcher below hands the pair to the runtime together with its kernel, and the pair then reads the kernel's own
// begin and end on the device clock (the interval a profiler reports for the dispatch), without changing what is
// enqueued.  Null (the default) launches plainly.
struct LaunchTimer { hipEvent_t start, stop; };
extern thread_local const LaunchTimer *launch_timer;

// phases: 1 = one kernel; 2 = a split-K operator (slice kernel, then the ordered finishing pass)
struct LaunchInfo { int workgroups; int threads; int lds_bytes; int wg_per_cu; const char *kernel; int phases; };

// phase 0 enqueues everything the operator needs; 1 only the slice / main kernel; 2 only the finishing pass
LaunchInfo launch_igemm(const GemmArgs &a, hipStream_t s, bool dry, int phase = 0);
LaunchInfo launch_dwconv(const StreamArgs &a, hipStream_t s, bool dry);
LaunchInfo launch_maxpool(const StreamArgs &a, hipStream_t s, bool dry);
LaunchInfo launch_gavgpool(const StreamArgs &a, hipStream_t s, bool dry);
LaunchInfo launch_eltwise(const StreamArgs &a, hipStream_t s, bool dry);   // affine / add / act / channel gate
LaunchInfo launch_concat(const StreamArgs &a, hipStream_t s, bool dry);
LaunchInfo launch_layernorm(const StreamArgs &a, hipStream_t s, bool dry);
LaunchInfo launch_softmax(const StreamArgs &a, hipStream_t s, bool dry);
// one wavefront that spins for `ticks` of the constant 100 MHz clock (stream placement probe)
void launch_spin(hipStream_t s, unsigned long long ticks);

}  // namespace gacer
