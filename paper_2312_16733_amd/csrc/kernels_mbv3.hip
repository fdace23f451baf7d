// Head of the MBV3-shaped SuperNet as one kernel: 3x3 stride-2 stem conv + SubnetNorm + hardswish, then the
// fixed first block (depthwise 3x3 + SubnetNorm + ReLU, pointwise 1x1 + SubnetNorm, residual), 3 -> 16 -> 16
// channels.  As separate launches this is four kernels (channel-padding copy, stem, depthwise, pointwise)
// that move the full-resolution 16-channel tensor through memory three times and each pay a launch's fixed
// cost; the arithmetic is 27 + 9 + 16 multiply-adds per output value, far too little for the matrix pipe to
// matter.  Here a block owns a 14 x 14 tile of the block's output: it stages the 33 x 33 x 3 input
// patch and all weights in LDS as fp32, computes the stem for the tile plus the depthwise conv's one-pixel halo
// (16 x 16 pixels; zeros outside the image, which is the depthwise conv's padding), keeps it in LDS rounded to
// bf16 exactly as the stored activation would be, and finishes the tile from there.  MH_PX adjacent pixels per
// thread share every weight read (the same LDS address in every lane); measured, one pixel per thread on 256
// threads is the fastest (48 us per launch at 160^2 and batch 64 against 70 us with two pixels on 128 threads and
// 119 us with four on 64: what counts is waves in flight, four blocks per CU at 100 VGPRs).  The loops over taps
// and input channels are kept rolled where full unrolling made the compiler request every weight ahead and
// run out of registers.  Every
// activation is rounded to bf16 where the unfused layers store it, sums are fp32 multiply-adds in a fixed
// order (taps row-major, channels innermost), so a request's values do not depend on its batch mates.
#include "common.h"

namespace sna {

constexpr int MH_T = 14;             // output tile side
constexpr int MH_G = MH_T + 2;       // with the halo: 16 x 16 stem pixels
constexpr int MH_P = 2 * MH_G + 1;   // input patch side (stride 2, 3 taps): 33
constexpr int MH_C = 16;             // channels of the stem and of the first block
constexpr int MH_PX = 1;             // adjacent pixels per thread (1, 2 or 4)
constexpr int MH_NT = MH_G * MH_G / MH_PX;   // threads per block: thread t owns row t / (16 / PX), columns PX (t % (16 / PX)) .. of the 16 x 16 grid

__device__ __forceinline__ void mh_unpack8(const uint4 v, float* f) {
  const unsigned u[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    f[2 * e] = __uint_as_float(u[e] << 16);
    f[2 * e + 1] = __uint_as_float(u[e] & 0xffff0000u);
  }
}
__device__ __forceinline__ uint4 mh_pack8(const float* f) {
  uint4 o;
  o.x = pack_bf16x2(f[0], f[1]); o.y = pack_bf16x2(f[2], f[3]);
  o.z = pack_bf16x2(f[4], f[5]); o.w = pack_bf16x2(f[6], f[7]);
  return o;
}

__global__ __launch_bounds__(MH_NT, 4) void mbv3_head_kernel(const Mbv3HeadArgs args) {
  __shared__ float patch[MH_P * MH_P * 3];
  __shared__ __attribute__((aligned(16))) float w0[27 * MH_C];     // stem: [(r * 3 + s) * 3 + c][k]
  __shared__ __attribute__((aligned(16))) float w1[9 * MH_C];      // depthwise: [r * 3 + s][c]
  __shared__ __attribute__((aligned(16))) float w2[MH_C * MH_C];   // pointwise: [c][k]
  __shared__ __attribute__((aligned(16))) float ss[6][MH_C];       // scale, shift of the three SubnetNorm layers
  __shared__ uint4 stem[MH_G * MH_G][2];                           // stem output of the tile and its halo, bf16

  const int g = find_problem(args, blockIdx.x);
  const Mbv3HeadProblem& p = args.p[g];
  int local = blockIdx.x - p.tile_start;
  const int tx = local % p.tiles_x; local /= p.tiles_x;
  const int ty = local % p.tiles_y;
  const int n = local / p.tiles_y;
  const int oh0 = ty * MH_T, ow0 = tx * MH_T;
  const int tid = threadIdx.x;

  // ---- input patch, weights and SubnetNorm vectors -> LDS (fp32).  The patch loads go out in two batches
  // per thread, each issued in full before its first value is used (one load at a time would pay the memory
  // round trip per element). ----
  {
    const int iy0 = 2 * oh0 - 3, ix0 = 2 * ow0 - 3;       // patch origin: rows 2 oh0 - 3 .., columns 2 ow0 - 3 ..
    const bf16_t* x = (const bf16_t*)p.x;
    const long img = (long)n * p.H * p.W;
    constexpr int NE = MH_P * MH_P * 3, PER = (NE + MH_NT - 1) / MH_NT, HALF = (PER + 1) / 2;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      bf16_t pv[HALF];
#pragma unroll
      for (int i = 0; i < HALF; ++i) {
        const int e = tid + (h * HALF + i) * MH_NT;
        const int pr = e / (MH_P * 3), rem = e - pr * (MH_P * 3), pc = rem / 3, c = rem - pc * 3;
        const int ih = iy0 + pr, iw = ix0 + pc;
        const bool ok = e < NE && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;      // zeros outside the image
        pv[i] = ok ? x[(img + (long)ih * p.W + iw) * p.pix_e + c] : (bf16_t)0;
      }
#pragma unroll
      for (int i = 0; i < HALF; ++i) {
        const int e = tid + (h * HALF + i) * MH_NT;
        if (e < NE) patch[e] = bf16_to_f32(pv[i]);
      }
    }
    // weights and SubnetNorm vectors: fixed trip counts, fully unrolled, so that the loads go out together
    const bf16_t* ws = (const bf16_t*)p.w_stem;
    constexpr int N0 = (27 * MH_C + MH_NT - 1) / MH_NT, N1 = (9 * MH_C + MH_NT - 1) / MH_NT, N2 = (MH_C * MH_C + MH_NT - 1) / MH_NT;
    bf16_t v0[N0], v1[N1], v2[N2];
#pragma unroll
    for (int i = 0; i < N0; ++i) {
      const int e = tid + i * MH_NT;
      const int k = e & 15, tc = e >> 4, tap = tc / 3, c = tc - tap * 3, r = tap / 3, sx = tap - r * 3;
      v0[i] = e < 27 * MH_C ? ws[(long)k * p.wk0 + r * p.wr0 + sx * p.ws0 + c] : (bf16_t)0;
    }
#pragma unroll
    for (int i = 0; i < N1; ++i) {
      const int e = tid + i * MH_NT;
      const int c = e & 15, tap = e >> 4, r = tap / 3, sx = tap - r * 3;
      v1[i] = e < 9 * MH_C ? ((const bf16_t*)p.w_dw)[r * p.wr1 + sx * p.ws1 + c] : (bf16_t)0;
    }
#pragma unroll
    for (int i = 0; i < N2; ++i) {
      const int e = tid + i * MH_NT;                         // [c = e / 16][k = e % 16]
      v2[i] = e < MH_C * MH_C ? ((const bf16_t*)p.w_pw)[(long)(e & 15) * p.wk2 + (e >> 4)] : (bf16_t)0;
    }
    float sv = 0.f;
    if (tid < 6 * MH_C) {
      const int v = tid >> 4;
      const float* src = v == 0 ? p.sc0 : v == 1 ? p.sh0 : v == 2 ? p.sc1 : v == 3 ? p.sh1 : v == 4 ? p.sc2 : p.sh2;
      sv = src[tid & 15];
    }
#pragma unroll
    for (int i = 0; i < N0; ++i)
      if (tid + i * MH_NT < 27 * MH_C) w0[tid + i * MH_NT] = bf16_to_f32(v0[i]);
#pragma unroll
    for (int i = 0; i < N1; ++i)
      if (tid + i * MH_NT < 9 * MH_C) w1[tid + i * MH_NT] = bf16_to_f32(v1[i]);
#pragma unroll
    for (int i = 0; i < N2; ++i)
      if (tid + i * MH_NT < MH_C * MH_C) w2[tid + i * MH_NT] = bf16_to_f32(v2[i]);
    if (tid < 6 * MH_C) ss[tid >> 4][tid & 15] = sv;
  }
  __syncthreads();

  static_assert(6 * MH_C <= MH_NT, "one SubnetNorm value per thread");
  const int gy = tid / (MH_G / MH_PX), gx0 = (tid % (MH_G / MH_PX)) * MH_PX;   // this thread's row and first column of the 16 x 16 grid

  // ---- stem for grid pixels (gy, gx0 ..) ----
  {
    float acc[MH_PX][MH_C];
#pragma unroll
    for (int j = 0; j < MH_PX; ++j)
#pragma unroll
      for (int k = 0; k < MH_C; ++k) acc[j][k] = 0.f;
#pragma unroll 1
    for (int r = 0; r < 3; ++r) {
      // the patch columns the thread's pixels' taps of this row touch
      float xr[2 * MH_PX + 1][3];
      const float* px = patch + ((2 * gy + r) * MH_P + 2 * gx0) * 3;
#pragma unroll
      for (int i = 0; i < (2 * MH_PX + 1) * 3; ++i) xr[i / 3][i % 3] = px[i];
#pragma unroll
      for (int s = 0; s < 3; ++s)
#pragma unroll
        for (int c = 0; c < 3; ++c) {
          const float4* wr = (const float4*)(w0 + ((r * 3 + s) * 3 + c) * MH_C);
#pragma unroll
          for (int k4 = 0; k4 < 4; ++k4) {
            const float4 w = wr[k4];
#pragma unroll
            for (int j = 0; j < MH_PX; ++j) {
              const float xv = xr[2 * j + s][c];
              acc[j][4 * k4 + 0] = fmaf(xv, w.x, acc[j][4 * k4 + 0]); acc[j][4 * k4 + 1] = fmaf(xv, w.y, acc[j][4 * k4 + 1]);
              acc[j][4 * k4 + 2] = fmaf(xv, w.z, acc[j][4 * k4 + 2]); acc[j][4 * k4 + 3] = fmaf(xv, w.w, acc[j][4 * k4 + 3]);
            }
          }
          if (c == 2) __builtin_amdgcn_sched_barrier(0);
        }
    }
    const int pp = oh0 - 1 + gy;
#pragma unroll
    for (int j = 0; j < MH_PX; ++j) {
      const int q = ow0 - 1 + gx0 + j;
      const bool inside = pp >= 0 && pp < p.Ho && q >= 0 && q < p.Wo;
      float v[MH_C];
#pragma unroll
      for (int k = 0; k < MH_C; ++k) v[k] = inside ? apply_act(fmaf(acc[j][k], ss[0][k], ss[1][k]), SNA_ACT_HSWISH) : 0.f;
      stem[gy * MH_G + gx0 + j][0] = mh_pack8(v);
      stem[gy * MH_G + gx0 + j][1] = mh_pack8(v + 8);
    }
  }
  __syncthreads();

  // ---- depthwise 3x3 + SubnetNorm + ReLU, pointwise + SubnetNorm + residual for output pixels (gy, gx0 ..)
  // of the 14 x 14 tile (grid pixel + 1) ----
  if (gy >= MH_T || gx0 >= MH_T || oh0 + gy >= p.Ho) return;
  float d[MH_PX][MH_C], centre[MH_PX][MH_C];
  {
    float acc1[MH_PX][MH_C];
#pragma unroll
    for (int j = 0; j < MH_PX; ++j)
#pragma unroll
      for (int c = 0; c < MH_C; ++c) acc1[j][c] = 0.f;
#pragma unroll 1
    for (int r = 0; r < 3; ++r) {
#pragma unroll
      for (int col = 0; col < MH_PX + 2; ++col) {            // the grid columns the thread's pixels' taps of this row touch
        const int gcol = gx0 + col < MH_G ? gx0 + col : MH_G - 1;     // (columns past the grid belong to pixels that are not stored)
        float xv[MH_C];
        mh_unpack8(stem[(gy + r) * MH_G + gcol][0], xv);
        mh_unpack8(stem[(gy + r) * MH_G + gcol][1], xv + 8);
#pragma unroll
        for (int s = 0; s < 3; ++s) {
          const int j = col - s;                             // pixel j takes this column as tap s
          if (j < 0 || j >= MH_PX) continue;
          const float4* wr = (const float4*)(w1 + (r * 3 + s) * MH_C);
#pragma unroll
          for (int c4 = 0; c4 < 4; ++c4) {
            const float4 w = wr[c4];
            acc1[j][4 * c4 + 0] = fmaf(xv[4 * c4 + 0], w.x, acc1[j][4 * c4 + 0]); acc1[j][4 * c4 + 1] = fmaf(xv[4 * c4 + 1], w.y, acc1[j][4 * c4 + 1]);
            acc1[j][4 * c4 + 2] = fmaf(xv[4 * c4 + 2], w.z, acc1[j][4 * c4 + 2]); acc1[j][4 * c4 + 3] = fmaf(xv[4 * c4 + 3], w.w, acc1[j][4 * c4 + 3]);
          }
          if (r == 1 && s == 1) {
#pragma unroll
            for (int c = 0; c < MH_C; ++c) centre[j][c] = xv[c];
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int j = 0; j < MH_PX; ++j)
#pragma unroll
      for (int c = 0; c < MH_C; ++c) d[j][c] = bf16_to_f32(f32_to_bf16(fmaxf(fmaf(acc1[j][c], ss[2][c], ss[3][c]), 0.f)));
  }
  float acc2[MH_PX][MH_C];
#pragma unroll
  for (int j = 0; j < MH_PX; ++j)
#pragma unroll
    for (int k = 0; k < MH_C; ++k) acc2[j][k] = 0.f;
#pragma unroll 4
  for (int c = 0; c < MH_C; ++c) {
    const float4* wr = (const float4*)(w2 + c * MH_C);
#pragma unroll
    for (int k4 = 0; k4 < 4; ++k4) {
      const float4 w = wr[k4];
#pragma unroll
      for (int j = 0; j < MH_PX; ++j) {
        acc2[j][4 * k4 + 0] = fmaf(d[j][c], w.x, acc2[j][4 * k4 + 0]); acc2[j][4 * k4 + 1] = fmaf(d[j][c], w.y, acc2[j][4 * k4 + 1]);
        acc2[j][4 * k4 + 2] = fmaf(d[j][c], w.z, acc2[j][4 * k4 + 2]); acc2[j][4 * k4 + 3] = fmaf(d[j][c], w.w, acc2[j][4 * k4 + 3]);
      }
    }
    __builtin_amdgcn_sched_barrier(0);       // keeps the weight reads of later channels from being requested (and held) ahead
  }
  const int oh = oh0 + gy;
#pragma unroll
  for (int j = 0; j < MH_PX; ++j) {
    const int ow = ow0 + gx0 + j;
    if (gx0 + j >= MH_T || ow >= p.Wo) break;
    float o[MH_C];
#pragma unroll
    for (int k = 0; k < MH_C; ++k) o[k] = fmaf(acc2[j][k], ss[4][k], ss[5][k]) + centre[j][k];
    uint4* y = (uint4*)((bf16_t*)p.y + (((long)n * p.Ho + oh) * p.Wo + ow) * MH_C);
    y[0] = mh_pack8(o);
    y[1] = mh_pack8(o + 8);
  }
}

int mbv3_head_channels() { return MH_C; }

hipError_t launch_mbv3_head(const Mbv3HeadArgs& a, hipStream_t s) {
  if (a.n == 0) return hipSuccess;
  Mbv3HeadArgs b = a;
  long start = 0;
  for (int i = 0; i < b.n; ++i) {
    Mbv3HeadProblem& p = b.p[i];
    if (p.N < 1 || p.H < 1 || p.W < 1 || p.Ho != (p.H - 1) / 2 + 1 || p.Wo != (p.W - 1) / 2 + 1 || p.pix_e < 3 ||
        !p.x || !p.y || !p.w_stem || !p.w_dw || !p.w_pw || !p.sc0 || !p.sh0 || !p.sc1 || !p.sh1 || !p.sc2 || !p.sh2)
      return hipErrorInvalidValue;
    p.tiles_x = (p.Wo + MH_T - 1) / MH_T; p.tiles_y = (p.Ho + MH_T - 1) / MH_T;
    p.tile_start = (int)start;
    p.tiles = p.N * p.tiles_x * p.tiles_y;
    start += p.tiles;
    if (start > 0x7fffffff) return hipErrorInvalidValue;
  }
  hipLaunchKernelGGL(mbv3_head_kernel, dim3((unsigned)start), dim3(MH_NT), 0, s, b);
  return hipGetLastError();
}

}  // namespace sna
