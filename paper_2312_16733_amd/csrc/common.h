// Internal declarations shared by the HIP kernels and the host-side planner.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/subnetact.h"

namespace sna {

typedef unsigned short bf16_t;   // raw bfloat16 bits

enum KClass {
  KC_IGEMM = 0,      // sliced implicit-GEMM conv / linear on bf16 MFMA
  KC_DIRECT = 1,     // direct conv (stems, fp32 tiny net)
  KC_DEPTHWISE = 2,
  KC_POOL = 3,       // max pool, global average pool
  KC_SE = 4,         // squeeze-excite gate + channel scale
  KC_LAYERNORM = 5,
  KC_ATTENTION = 6,
  KC_COPY = 7,       // request gather / logits scatter
  KC_FOLD = 8,       // SubnetNorm statistics folding (load time)
  KC_KREDUCE = 9,    // sum of the K-chunk partials + fused epilogue of a split igemm
  KC_STEMPOOL = 10,  // fused 7x7/2 stem conv + SubnetNorm + ReLU + 3x3/2 max pool
  KC_CALIB = 11,     // SubnetNorm calibration: channel statistics and the normalise pass
  KC_COUNT = 12
};

// ---- one problem of a grouped launch -------------------------------------------------------
// A grouped launch carries up to SNA_MAX_GROUPS problems by value in the kernel
// arguments; block b belongs to the problem whose [tile_start, tile_start + tiles)
// range holds b.  One problem = one layer of one subnet cfg over that cfg's requests.

struct ConvProblem {
  const void* x;        // [N][H][W][C] activations (active channels, dense)
  const void* w;        // max-size weights, already offset to the centre window's first tap
  const float* scale;   // [K] or nullptr (= 1)
  const float* shift;   // [K] or nullptr (= 0)
  const void* res;      // [N][Ho][Wo][K] residual or nullptr
  void* y;              // [N][Ho][Wo][K]
  int N, H, W, C;       // C = active input channels
  int Ho, Wo, K;        // K = active output channels
  int R, S, stride, pad;
  int wk, wr, ws;       // element strides of the stored weight tensor (c stride = 1)
  int M;                // N*Ho*Wo
  int C8, K8;           // C/8, R*S*C/8 (igemm only)
  unsigned magic_wo, magic_ho;   // floor(2^32 / d) + 1 for d = Wo, Ho (0 when d == 1): x / d = mulhi(x, magic) while x * d < 2^32
  int inv_s;            // ceil(2^16 / S): tap row r = (rs * inv_s) >> 16
  int tiles_n;          // tiles along K (igemm)
  int tile_start, tiles;
  int act;              // sna_act
  int out_fp32;         // 1: y is float (logits), else storage dtype
  int y_stride;         // elements between output rows (>= K); lets a linear write a column block
  int res_stride;
  unsigned x_bytes, w_bytes;   // extent of x and of the active weight rows, for bounds-checked loads
  int c_count;          // host bookkeeping: input channels that count as algorithmic work (0 = C)
  int res_after_act;    // 0: y = act(norm(conv) + res); 1: y = act(norm(conv)) + res
  // K chunking (igemm).  The reduction is cut into chunks of kt_chunk steps of 64 elements, a
  // function of the layer's active shape only; chunk sums are added in order in fp32.  Either one
  // block walks all chunks (parts = 1, kt_part >= all steps) or each chunk gets its own blocks
  // (parts = number of chunks, kt_part = kt_chunk) that write raw fp32 sums for the reduction kernel.
  int parts, tiles_base;         // tiles = parts * tiles_base
  int kt_part, kt_chunk;
  unsigned long part_stride;     // bytes between the parts' fp32 outputs
  // Reduction inside the matrix kernel (parts > 1, counters != nullptr): every block writes its raw fp32
  // chunk sum to part_buf ([parts][M][K], part_stride bytes apart) and bumps its tile's counter; the block
  // that arrives last adds the parts in chunk order and finishes the layer (scale, shift, res, act, y as
  // for parts == 1), then puts the counter back to zero.  With counters == nullptr and parts > 1 the
  // kernel writes the raw sums to y and splitk_reduce_kernel finishes the layer in a second launch.
  float* part_buf;
  int* counters;                 // [tiles_base] zero-initialised ints of this problem
};

struct ConvGroupArgs {
  int n;
  int total_tiles;      // sum of tiles over the problems
  ConvProblem p[SNA_MAX_GROUPS];
};

struct PoolProblem {    // max pool 3x3/2 or global average pool
  const void* x; void* y;
  int N, H, W, C, Ho, Wo;
  int out_fp32;         // global average pool only: write fp32 instead of the storage dtype
  int tile_start, tiles;
};
struct PoolGroupArgs { int n; PoolProblem p[SNA_MAX_GROUPS]; };

struct DwProblem {
  const void* x; const void* w; const float* scale; const float* shift; void* y;
  int N, H, W, C, Ho, Wo;
  int k, stride, pad;
  int wr, ws;           // element strides of the stored [R][S][C_max] kernel
  int act;
  // Squeeze-excite pool fused into the layer: the grid is laid out per request (bpr blocks each) and
  // every block writes the sums of its own outputs, as stored, per channel: pool_part[n][block][C].
  float* pool_part;     // nullptr: flat grid, no pool
  int bpr;
  int raw_out;          // calibration: y is fp32 and gets the bare sums (no SubnetNorm, no activation)
  int tile_start, tiles;
};
struct DwGroupArgs { int n; DwProblem p[SNA_MAX_GROUPS]; };

struct SeProblem {
  const void* x;        // [N][HW][C] depthwise output
  void* y;              // gated output (may alias x)
  const void* w1; const float* b1;  // [Q_max][C_max] stored; leading [Q][C] used
  const void* w2; const float* b2;  // [C_max][Q_max]
  float* pooled;        // [N][pool_segs][C] partial sums of the pool, written by the depthwise kernel's blocks
  float* hidden;        // [N][Q] scratch
  int N, HW, C, Q;
  int w1_stride, w2_stride;
  int pool_segs;        // partial sums per request, added in order and scaled by inv_hw
  float inv_hw;
  int tile_start, tiles;
};
struct SeGroupArgs { int n; SeProblem p[SNA_MAX_GROUPS]; };

struct LnProblem {
  const void* x; const float* gamma; const float* beta; void* y;
  int rows, cols;
  int tile_start, tiles;
};
struct LnGroupArgs { int n; LnProblem p[SNA_MAX_GROUPS]; };

struct AttnProblem {
  const void* q; const void* k; const void* v; void* o;   // [B][S][heads*64], row stride ld
  int B, S, heads, ld;
  int tile_start, tiles;
};
struct AttnGroupArgs { int n; AttnProblem p[SNA_MAX_GROUPS]; };

// fused ResNet stem (7x7 stride-2 conv, SubnetNorm, ReLU, 3x3 stride-2 max pool)
struct StemPoolProblem {
  const void* x;        // request images: [N][H][W][8] channel-padded copy, or the caller's [N][H][W][3] (see pix_b)
  const void* w;        // stem weights stored with 8 input channels, first tap of the 7x7 window
  const float* scale; const float* shift;
  void* y;              // [N][Po][Qo][K]
  int N, H, W;
  int Ho, Wo;           // conv output
  int Po, Qo;           // pooled output
  int K;                // active out channels (multiple of 8, <= 64)
  int wk, wr, ws;       // element strides of the stored weight tensor
  unsigned x_bytes;
  int pix_b;            // bytes between input pixels: 16 for the padded copy, 6 for a 3-channel image read in place
  int tiles_x, tiles_y; // pooled 4 x 16 tiles per image
  int tile_start, tiles;
};
struct StemPoolArgs { int n; int total_tiles; StemPoolProblem p[SNA_MAX_GROUPS]; };

// Head of the MBV3-shaped SuperNet in one launch: stem 3x3/2 (3 -> 16) + SubnetNorm + hardswish, depthwise 3x3 +
// SubnetNorm + ReLU, pointwise 16 -> 16 + SubnetNorm, residual.
struct Mbv3HeadProblem {
  const void* x;        // request images [N][H][W][pix_e], channels 0..2 used
  void* y;              // [N][Ho][Wo][16]
  const void* w_stem; const void* w_dw; const void* w_pw;   // first tap / first element of the slices
  const float *sc0, *sh0, *sc1, *sh1, *sc2, *sh2;           // folded SubnetNorm of the three layers
  int N, H, W, Ho, Wo;
  int pix_e;            // elements between input pixels: 3 for images read in place, 8 for the channel-padded copy
  int wk0, wr0, ws0;    // element strides of the stored stem weights (out channel, tap row, tap column)
  int wr1, ws1;         // depthwise kernel: tap row, tap column
  int wk2;              // pointwise weights: out channel
  int tiles_x, tiles_y; // 14 x 14 output tiles per image (filled by the launcher)
  int tile_start, tiles;
};
struct Mbv3HeadArgs { int n; Mbv3HeadProblem p[SNA_MAX_GROUPS]; };

struct CopyItem { unsigned long src, dst; unsigned long n; };   // byte offsets / length (even)
#define SNA_COPY_ITEMS 128
struct CopyArgs { const void* src; void* dst; int n; CopyItem it[SNA_COPY_ITEMS]; };

// request inputs [pixels][c_in] bf16 -> [pixels][8] bf16, zero-padded channels (also gathers requests)
struct PadItem { unsigned long src, dst; unsigned long pixels; };   // byte offsets
#define SNA_PAD_ITEMS 128
struct PadArgs { const void* src; void* dst; int n; int c_in; PadItem it[SNA_PAD_ITEMS]; };

// SubnetNorm calibration of one layer: per-channel mean and population variance of its raw conv output
// [M][K] fp32 over the M rows (all requests, all pixels), written into the caller's statistics table
// (fp32) and folded into this layer's scale / shift from the values as stored.
struct NormCalArgs {
  const float* raw; int M, K;
  float* part; int nrb;            // [nrb][K][3] (count, mean, M2) of row blocks of SNA_CAL_ROWS rows
  float* mean; float* var;         // rows of the statistics table, at this layer's offset
  const float* gamma; const float* beta;
  float* scale; float* shift;      // folded table, same offset
};
#define SNA_CAL_ROWS 256
// y = act(scale * raw + shift (+ res)) in the family's storage dtype: what the fused epilogues do, on the
// raw conv output kept by a calibration pass
struct NormApplyArgs {
  const float* raw; const float* scale; const float* shift; const void* res; void* y;
  int M, K, act, res_after_act, res_stride, y_stride;
};

// fp32 partial sums of split reductions: fixed region at the end of the workspace
constexpr size_t kPartialBytes = (size_t)64 << 20;
// tile counters of reductions that finish inside the matrix kernel: one per output tile of every such
// problem in one launch
constexpr size_t kTileCounters = 16384;

// ---- launchers (defined in the .hip files) ---------------------------------------------------
hipError_t launch_igemm(const ConvGroupArgs& a, int variant, bool chunked, hipStream_t s);
bool igemm_variant_ok(int variant, const ConvProblem& p);   // can this tile variant run this problem (some take 3x3 stride-1 layers only)
hipError_t launch_splitk_reduce(const ConvGroupArgs& a, hipStream_t s);
hipError_t launch_stem_pool(const StemPoolArgs& a, hipStream_t s);
hipError_t launch_mbv3_head(const Mbv3HeadArgs& a, hipStream_t s);
int mbv3_head_channels();                          // the width launch_mbv3_head is built for
void igemm_tile_shape(int variant, int* bm, int* bn);
int igemm_num_variants();
hipError_t launch_direct_conv(const ConvGroupArgs& a, int dtype, hipStream_t s);
hipError_t launch_maxpool(const PoolGroupArgs& a, int dtype, hipStream_t s);
hipError_t launch_gap(const PoolGroupArgs& a, int dtype, hipStream_t s);
hipError_t launch_depthwise(const DwGroupArgs& a, hipStream_t s);
hipError_t launch_norm_calibrate(const NormCalArgs& a, hipStream_t s);
hipError_t launch_norm_apply(const NormApplyArgs& a, int dtype, hipStream_t s);
int depthwise_pool_blocks(int Ho, int Wo, int C);   // blocks per request of a depthwise layer with the fused pool
hipError_t launch_se(const SeGroupArgs& a, hipStream_t s);
hipError_t launch_layernorm(const LnGroupArgs& a, hipStream_t s);
hipError_t launch_attention(const AttnGroupArgs& a, hipStream_t s);
hipError_t launch_copy(const CopyArgs& a, hipStream_t s);
hipError_t launch_pad_input(const PadArgs& a, hipStream_t s);
hipError_t launch_fold_stats(const float* stats, float* folded, int n_subnets, long row_len, hipStream_t s);

// ---- device helpers ---------------------------------------------------------------------------
#if defined(__HIPCC__)
__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((unsigned)v) << 16); }
// round-to-nearest-even through the hardware conversion (v_cvt_pk_bf16_f32); checked bit for bit
// against the integer formulation on all finite patterns
typedef __bf16 sna_bf16x2 __attribute__((ext_vector_type(2)));
typedef float sna_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
  const sna_f32x2 v = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, sna_bf16x2));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }
// Standard normal CDF Phi(v) = erfc(-v / sqrt 2) / 2 for the exact (erf) GELU.  erfc of a non-negative
// argument by the five-term rational formula of Abramowitz & Stegun 7.1.26 (absolute error
// < 1.5e-7, the level of fp32 rounding), evaluated on |v| so that the negative tail has no
// cancellation: about a dozen instructions against the library erff's branchy several dozen, which
// showed as 6-10 us per FFN launch of 8192 x 3072 outputs.
__device__ __forceinline__ float normal_cdf(float v) {
  const float x = fabsf(v) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.f));
  float poly = fmaf(1.061405429f, t, -1.453152027f);
  poly = fmaf(poly, t, 1.421413741f);
  poly = fmaf(poly, t, -0.284496736f);
  poly = fmaf(poly, t, 0.254829592f);
  const float q = 0.5f * poly * t * __builtin_amdgcn_exp2f(-x * x * 1.44269504088896340736f);
  return v < 0.f ? q : 1.f - q;
}
__device__ __forceinline__ float apply_act(float v, int act) {
  if (act == SNA_ACT_RELU) return fmaxf(v, 0.f);
  if (act == SNA_ACT_HSWISH) return v * fminf(fmaxf(v + 3.f, 0.f), 6.f) * (1.f / 6.f);
  if (act == SNA_ACT_GELU) return v * normal_cdf(v);
  return v;
}
// problem lookup for a grouped launch: linear scan over <= 16 entries (uniform per block)
template <class Args>
__device__ __forceinline__ int find_problem(const Args& a, int b) {
  int g = 0;
#pragma unroll 1
  for (int i = 1; i < a.n; ++i)
    if (b >= a.p[i].tile_start) g = i;
  return g;
}
#endif

}  // namespace sna
