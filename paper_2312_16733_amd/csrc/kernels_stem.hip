// ResNet stem in one kernel: 7x7 stride-2 WeightSlice conv over the request image (read in place, or a
// channel-padded copy of scattered requests),
// SubnetNorm scale/shift, ReLU and the 3x3 stride-2 max pool that follows it.  (WeightSlice and
// SubnetNorm operators of the paper's section "SubNetAct: Instantaneous Model Actuation": the block
// reads the leading K_active output channels of the resident 7x7 stem tensor in place and applies the
// subnet's own folded statistics.)
//
// The generic implicit GEMM gathers the stem's 49 taps per output pixel through the texture path
// (16 bytes each) and writes a full-resolution activation that the pool reads straight back; here
// a block stages the input patch of a pooled tile in LDS once, runs the MFMAs out of LDS, keeps the
// conv output of the tile in LDS and writes only the pooled result: the input is read once (plus
// halo), the conv output never touches HBM.
//
// Geometry of one tile: PH x PW = 4 x 16 pooled pixels <- (2 PH + 1) x (2 PW + 1) = 9 x 33 conv
// pixels (the pool's window with its halo; a neighbouring tile recomputes the shared row / column,
// 16 % extra MFMA work) <- 23 x 71 input pixels, kept in LDS as 4 channels (8 bytes: 3 + a zero) each.
// The window of a conv pixel starts at an even column of the patch (stride 2), so a 16-byte unit of
// LDS is a pair of horizontally adjacent taps: the reduction runs over 7 window rows x 4 column
// pairs = 28 units of 8 elements (the eighth column has zero weights), 224 instead of the 392 that
// one tap per unit with channels padded to 8 would take.
// MFMA shape: rows = conv pixels of the tile in raster order (297, ten 32-row tiles over 4 waves),
// columns = output channels (<= 64), reduction = 28 units x 8 elements, two units per MFMA.
// Blocks are persistent: weights, scale and shift go to LDS once per problem, then the block walks
// its tiles; the next tile's patch is requested as soon as the MFMAs are done with the current one.
// The conv tile is staged over the patch (free by then), which keeps a block at 76 KB of LDS: two
// blocks per CU, so one block's MFMAs run under the other's epilogue and pool.
#include "common.h"

#include <atomic>

namespace sna {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((address_space(3))) char lds_char;

namespace stem {
constexpr int KS = 7, PAIRS = 4, SLOTS = KS * PAIRS;                    // units of the reduction: (window row, column pair)
[[maybe_unused]] constexpr int NSLICE = SLOTS / 2;                     // device code only
constexpr int PH = 4, PW = 16;
constexpr int SH = 2 * PH + 1, SW = 2 * PW + 1, NSP = SH * SW;          // conv pixels per tile: 9 x 33 = 297
constexpr int IH = 2 * SH + 5, IW = 2 * SW + 5, NIP = IH * IW;          // input pixels per tile: 23 x 71 = 1633
constexpr int ROW_TILES = (NSP + 31) / 32;                              // 10
constexpr int IWP = (IW + 1) / 2;                                       // 36 column pairs per patch row
constexpr int NIS = IH * IWP * 2;                                       // pixel slots of a patch incl. the spare last column: 1656
constexpr int PASSES = (NIS + 255) / 256;                               // 7 passes of 256 pixels
constexpr int KMAX = 64;
constexpr int W_ROW_B = SLOTS * 16 + 16;                                // one out channel's taps in LDS; the pad spreads rows over banks
constexpr int OFF_W = 0;
constexpr int OFF_PATCH = OFF_W + KMAX * W_ROW_B;                       // 29696
constexpr int OFF_SOUT = OFF_PATCH;                                     // the conv tile is staged over the patch, free by then
constexpr int SOUT_ROW_B = KMAX * 2 + 16;                               // one conv pixel: 64 bf16 + pad against bank conflicts
constexpr int PATCH_B = PASSES * 256 * 8, SOUT_B = ROW_TILES * 32 * SOUT_ROW_B;
constexpr int OFF_SS = OFF_PATCH + (PATCH_B > SOUT_B ? PATCH_B : SOUT_B);   // + 46080
constexpr int SMEM = OFF_SS + 2 * KMAX * 4;
static_assert(2 * SMEM <= 160 * 1024, "two blocks per CU");
static_assert((SW - 1) + PAIRS - 1 < IWP && 2 * (SH - 1) + KS - 1 < IH, "fragment reads stay inside the patch");
static_assert((2 * (PH - 1) + 2) * SW + 2 * (PW - 1) + 2 < NSP, "pool windows stay inside the conv tile");
}  // namespace stem

// TWO: some problem of the launch has more than 32 output channels (second 32-channel column tile).
template <bool TWO>
__global__ __launch_bounds__(256, 2) void stem_pool_kernel(const StemPoolArgs args) {
#if defined(__HIP_DEVICE_COMPILE__)        // the host pass needs the symbol only, not the body
  using namespace stem;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char* const w_lds = smem + OFF_W;
  char* const patch = smem + OFF_PATCH;
  char* const sout = smem + OFF_SOUT;
  float* const ss = (float*)(smem + OFF_SS);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, l32 = lane & 31;

  // this lane's conv pixels (one per row tile it computes) and their first input pixel in the patch
  int pbase[3];
#pragma unroll
  for (int i = 0; i < 3; ++i) {
    const int sp = 32 * (wave + 4 * i) + l32;              // waves 2 and 3 have no third row tile: they redo pixel 0
    const int spc = sp < NSP ? sp : 0;
    const int sy = spc / SW, sx = spc - sy * SW;
    pbase[i] = ((2 * sy) * IWP + sx) * 16;
  }

  // which input pixel of a patch each of this thread's DMA lanes fetches (the same for every tile)
  int lane_yx[PASSES];
#pragma unroll
  for (int pass = 0; pass < PASSES; ++pass) {
    const int i = pass * 256 + tid;                          // pixel slot: row-major, 2 IWP slots per row
    const int iy = i / (2 * IWP), ix = i - iy * (2 * IWP);
    lane_yx[pass] = (i < NIS && ix < IW) ? (iy << 16) | ix : -1;     // the spare column past the patch stays zero
  }

  // The input patch of a tile goes through registers: three channel loads per pixel at the image's own
  // pixel stride (so a 3-channel request image is read in place, no padded copy), zeros outside the
  // image; store_patch() then writes 8 bytes per pixel (3 channels and a zero) where the MFMAs expect them.
  unsigned pk[PASSES][2];
  auto load_patch = [&](int t) {
    const int gp = find_problem(args, t);
    const StemPoolProblem& q = args.p[gp];
    const int local = t - q.tile_start;
    const int per_img = q.tiles_x * q.tiles_y;
    const int n = local / per_img;
    const int rem = local - n * per_img;
    const int ty = rem / q.tiles_x, tx = rem - ty * q.tiles_x;
    const int iy0 = 2 * (2 * ty * PH - 1) - 3, ix0 = 2 * (2 * tx * PW - 1) - 3;      // first input pixel of the patch
    // bounds-checked 2-byte loads at 32-bit offsets: a pixel outside the image gets an out-of-range
    // offset, which reads as zero (the padding)
    const __amdgpu_buffer_rsrc_t rsrc_x = __builtin_amdgcn_make_buffer_rsrc((void*)q.x, 0, (int)q.x_bytes, 0x00020000);
    const int row_b = q.W * q.pix_b;
    const int base = (n * q.H + iy0) * row_b + ix0 * q.pix_b;       // may be negative; only used where ok
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass) {
      const int ly = lane_yx[pass] >> 16, lx = lane_yx[pass] & 0xffff;
      const int gy = iy0 + ly, gx = ix0 + lx;
      const bool ok = lane_yx[pass] >= 0 && gy >= 0 && gy < q.H && gx >= 0 && gx < q.W;
      const int off = ok ? base + ly * row_b + lx * q.pix_b : (int)0x80000000;
      const unsigned c0 = __builtin_amdgcn_raw_buffer_load_b16(rsrc_x, off, 0, 0);
      const unsigned c1 = __builtin_amdgcn_raw_buffer_load_b16(rsrc_x, off + 2, 0, 0);
      const unsigned c2 = __builtin_amdgcn_raw_buffer_load_b16(rsrc_x, off + 4, 0, 0);
      pk[pass][0] = c0 | (c1 << 16);
      pk[pass][1] = c2;
    }
  };
  auto store_patch = [&]() {
#pragma unroll
    for (int pass = 0; pass < PASSES; ++pass)
      *(uint2*)(patch + (pass * 256 + tid) * 8) = make_uint2(pk[pass][0], pk[pass][1]);
  };

  int cur_g = -1;
  if ((int)blockIdx.x < args.total_tiles) { load_patch(blockIdx.x); store_patch(); }
  for (int tile = blockIdx.x; tile < args.total_tiles; tile += gridDim.x) {
    const int g = find_problem(args, tile);
    const StemPoolProblem& p = args.p[g];
    const int K = p.K;
    if (g != cur_g) {
      // the barrier that ends every tile guarantees that no wave still reads w_lds or ss
      const bf16_t* w = (const bf16_t*)p.w;
      for (int i = tid; i < KMAX * SLOTS; i += 256) {
        const int k = i / SLOTS, slot = i - k * SLOTS;
        const int r = slot / PAIRS, c = 2 * (slot - r * PAIRS);          // taps (r, c) and (r, c + 1), 3 channels each
        uint4 v = make_uint4(0, 0, 0, 0);
        if (k < K) {
          const bf16_t* t0 = w + (long)k * p.wk + (long)r * p.wr + (long)c * p.ws;
          v.x = (unsigned)t0[0] | ((unsigned)t0[1] << 16);
          v.y = (unsigned)t0[2];
          if (c + 1 < KS) {
            const bf16_t* t1 = t0 + p.ws;
            v.z = (unsigned)t1[0] | ((unsigned)t1[1] << 16);
            v.w = (unsigned)t1[2];
          }
        }
        *(uint4*)(w_lds + k * W_ROW_B + slot * 16) = v;
      }
      if (tid < KMAX) {
        ss[tid] = tid < K ? p.scale[tid] : 0.f;
        ss[KMAX + tid] = tid < K ? p.shift[tid] : 0.f;
      }
      cur_g = g;
    }
    const int local = tile - p.tile_start;
    const int per_img = p.tiles_x * p.tiles_y;
    const int n = local / per_img;
    const int rem = local - n * per_img;
    const int ty = rem / p.tiles_x, tx = rem - ty * p.tiles_x;
    const int py0 = ty * PH, px0 = tx * PW;
    const int sy0 = 2 * py0 - 1, sx0 = 2 * px0 - 1;          // first conv pixel of the tile (may be -1)

    __syncthreads();                                         // patch, weights, scale / shift visible to all

    // ---- MFMAs out of LDS ---------------------------------------------------------------------
    // No branches in this loop (a wave without a third row tile recomputes pixel 0 and drops it), so
    // that the fragment reads of slice s + 1 can be issued ahead of the MFMAs of slice s.
    constexpr int TNJ = TWO ? 2 : 1;
    f32x16 acc[3][TNJ];
    u32x4 af[2][3], bf[2][TNJ];
    auto fetch = [&](int s, int buf) {
      const int slot = 2 * s + half;                         // (window row r, column pair jp)
      const int r = slot / PAIRS, jp = slot - r * PAIRS;
      const int aoff = (r * IWP + jp) * 16;                  // conv pixel sx, pair jp: patch columns 2 sx + 2 jp, + 1
#pragma unroll
      for (int j = 0; j < TNJ; ++j) bf[buf][j] = *(const u32x4*)(w_lds + (32 * j + l32) * W_ROW_B + slot * 16);
#pragma unroll
      for (int i = 0; i < 3; ++i) af[buf][i] = *(const u32x4*)(patch + pbase[i] + aoff);
    };
    fetch(0, 0);
#pragma unroll
    for (int s = 0; s < NSLICE; ++s) {
      const int cur = s & 1;
      if (s + 1 < NSLICE) fetch(s + 1, cur ^ 1);
#pragma unroll
      for (int i = 0; i < 3; ++i)
#pragma unroll
        for (int j = 0; j < TNJ; ++j) {
          if (s == 0) {
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bf[cur][j]),
                                                                __builtin_bit_cast(bf16x8, af[cur][i]), zero, 0, 0, 0);
          } else {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bf[cur][j]),
                                                                __builtin_bit_cast(bf16x8, af[cur][i]), acc[i][j], 0, 0, 0);
          }
        }
    }

    __syncthreads();                                         // every wave is done with the patch
    const bool more = tile + (int)gridDim.x < args.total_tiles;
    if (more) load_patch(tile + gridDim.x);                  // arrives under the epilogue and the pool

    // ---- SubnetNorm + ReLU, conv tile -> LDS as bf16 ------------------------------------------
    float4 sc[TNJ][4], sh[TNJ][4];
#pragma unroll
    for (int j = 0; j < TNJ; ++j)
#pragma unroll
      for (int gq = 0; gq < 4; ++gq) {
        sc[j][gq] = *(const float4*)(ss + 32 * j + 8 * gq + 4 * half);
        sh[j][gq] = *(const float4*)(ss + KMAX + 32 * j + 8 * gq + 4 * half);
      }
    // accumulator element v of lane l: channel 8*(v/4) + 4*(l/32) + v%4 of its column tile, pixel l%32
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      const int sp = 32 * (wave + 4 * i) + l32;
      const int sy = sp / SW, sx = sp - sy * SW;
      const int ay = sy0 + sy, ax = sx0 + sx;
      const bool valid = sp < NSP && ay >= 0 && ay < p.Ho && ax >= 0 && ax < p.Wo;
      if (sp >= ROW_TILES * 32) continue;                    // the third row tile of waves 2 and 3 does not exist
#pragma unroll
      for (int j = 0; j < TNJ; ++j) {
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          const int ch = 32 * j + 8 * gq + 4 * half;
          const float v0 = fmaxf(fmaf(acc[i][j][4 * gq + 0], sc[j][gq].x, sh[j][gq].x), 0.f);
          const float v1 = fmaxf(fmaf(acc[i][j][4 * gq + 1], sc[j][gq].y, sh[j][gq].y), 0.f);
          const float v2 = fmaxf(fmaf(acc[i][j][4 * gq + 2], sc[j][gq].z, sh[j][gq].z), 0.f);
          const float v3 = fmaxf(fmaf(acc[i][j][4 * gq + 3], sc[j][gq].w, sh[j][gq].w), 0.f);
          uint2 o;
          // after the ReLU every value is >= 0: with the sign bit cleared (-0 -> +0) bf16 order is
          // unsigned 16-bit order, and 0 can stand in for the pool's -inf padding
          o.x = valid ? (pack_bf16x2(v0, v1) & 0x7fff7fffu) : 0u;
          o.y = valid ? (pack_bf16x2(v2, v3) & 0x7fff7fffu) : 0u;
          *(uint2*)(sout + sp * SOUT_ROW_B + ch * 2) = o;
        }
      }
    }
    __syncthreads();                                         // conv tile complete

    // ---- 3x3 stride-2 max pool out of LDS, 16-byte stores -------------------------------------
    const int octs = K >> 3;
    for (int it = tid; it < PH * PW * octs; it += 256) {
      const int pp = it / octs, oct = it - pp * octs;
      const int ly = pp / PW, lx = pp - ly * PW;
      const int py = py0 + ly, px = px0 + lx;
      if (py >= p.Po || px >= p.Qo) continue;
      typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
      u16x2 best[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) best[e] = u16x2{0, 0};
#pragma unroll
      for (int dy = 0; dy < 3; ++dy)
#pragma unroll
        for (int dx = 0; dx < 3; ++dx) {
          const uint4 v = *(const uint4*)(sout + ((2 * ly + dy) * SW + 2 * lx + dx) * SOUT_ROW_B + oct * 16);
          const unsigned u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) best[e] = __builtin_elementwise_max(best[e], __builtin_bit_cast(u16x2, u[e]));
        }
      uint4 o;
      o.x = __builtin_bit_cast(unsigned, best[0]); o.y = __builtin_bit_cast(unsigned, best[1]);
      o.z = __builtin_bit_cast(unsigned, best[2]); o.w = __builtin_bit_cast(unsigned, best[3]);
      *(uint4*)((bf16_t*)p.y + (((long)n * p.Po + py) * p.Qo + px) * K + oct * 8) = o;
    }
    __syncthreads();                                         // every thread is done reading the conv tile, which lies over the patch
    if (more) store_patch();
    __syncthreads();                                         // the next tile's patch in place
  }
#endif
}

hipError_t launch_stem_pool(const StemPoolArgs& a, hipStream_t s) {
  if (a.n == 0 || a.total_tiles == 0) return hipSuccess;
  for (int i = 0; i < a.n; ++i) {
    const StemPoolProblem& p = a.p[i];
    if (p.K < 8 || p.K > stem::KMAX || p.K % 8 || p.tiles_x * stem::PW < p.Qo || p.tiles_y * stem::PH < p.Po ||
        p.tiles != p.N * p.tiles_x * p.tiles_y || p.pix_b < 6 || p.pix_b % 2 ||
        (size_t)p.N * p.H * p.W * p.pix_b > (size_t)p.x_bytes || p.x_bytes >= 0x80000000u)    // 32-bit offsets; 2^31 marks "outside"
      return hipErrorInvalidValue;
  }
  bool two = false;
  for (int i = 0; i < a.n; ++i) two = two || a.p[i].K > 32;
  void (*fn)(const StemPoolArgs) = two ? stem_pool_kernel<true> : stem_pool_kernel<false>;
  static std::atomic<bool> attr_done[2];      // handles on several threads may get here together
  if (!attr_done[two].load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, stem::SMEM);
    if (e != hipSuccess) return e;
    attr_done[two].store(true, std::memory_order_release);
  }
  const int blocks = a.total_tiles < 512 ? a.total_tiles : 512;     // two persistent blocks per CU
  hipLaunchKernelGGL(fn, dim3(blocks), dim3(256), stem::SMEM, s, a);
  return hipGetLastError();
}

}  // namespace sna
