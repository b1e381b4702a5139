// Depthwise 3x3 conv2d and the 1x1 conv2d behind it as one kernel (paper Section 4.1: the operators
// of one primitive function run in one kernel; Section 5.2: what each saved launch and each saved
// round trip through memory is worth).
//
// The two are the separable block of the MobileNet family.  Run as two kernels, the depthwise
// output goes to HBM and comes straight back as the activation operand of the 1x1 conv.  Here a
// workgroup owns a TH x TW rectangle of output pixels of one image and BN output channels, and
// walks the depthwise channels in chunks of CK:
//   1. the input patch under the rectangle, CK channels deep, comes in with global->LDS loads
//      (taps in the padding get an out-of-range offset and arrive as zeros);
//   2. the vector ALUs compute the depthwise outputs of the chunk from that patch (MH x MW outputs
//      x 8 channels per thread, fp32 accumulation, the same order of sums and the same fused
//      scale/shift/relu as the standalone depthwise kernels), narrow them to fp16 and write them into
//      LDS in the layout the matrix cores read their activation operand from;
//   3. the matrix cores multiply that tile with the chunk of 1x1 filters that has meanwhile arrived
//      in a two-stage LDS ring, as in the implicit-GEMM kernel.
// The fp16 narrowing in the middle is that of the two-kernel pipeline, and the 1x1 reduction runs
// in the same order with the same instruction, so the result equals the two launches bit for bit.
// A workgroup per tile of output channels recomputes the depthwise tile; with few output pixels
// (the deep layers) that is what buys enough workgroups to fill the chip.
#include <cstdio>

#include "dma_common.hpp"
#include "dw_math.hpp"

namespace relay {
namespace {

// Slot of patch pixel p (in units of one pixel's CV vectors).  Threads that read the same tap of
// neighbouring micro-tiles are MW*STRIDE pixels apart, a multiple of the LDS bank period; the XOR
// with a few higher bits of p spreads them over the banks.  An involution inside aligned groups of
// 16 pixels, so the loader applies the same function to find the pixel that belongs in a slot.
template <int CV>
__device__ __forceinline__ int patch_slot(int p) {
  return CV <= 4 ? p ^ ((p >> 2) & 3) : p ^ ((p >> 1) & 1);
}

// Workgroup barrier that the compiler does not move LDS accesses across (the waits that make this
// wave's own LDS writes and global->LDS loads complete stand in front of it at every use).
__device__ __forceinline__ void barrier_fenced() {
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

template <int STRIDE, int TH, int TW, int MH, int MW, int WAVES_M, int WAVES_N, int TM, int TN, int KP>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void dwpw_fused_kernel(const DwPwArgs a) {
  constexpr int NW = WAVES_M * WAVES_N, NT = 64 * NW;
  constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32, WTM = TM * 32, WTN = TN * 32;
  static_assert(TH * TW <= BM, "the rectangle must fit the rows of the tile");
  static_assert(TH % MH == 0 && TW % MW == 0, "whole micro-tiles");
  constexpr int CV = KP * BKV;                     // 16-byte channel vectors per pixel per chunk
  constexpr int CK = CV * 8;                       // depthwise channels per chunk
  constexpr int PH = (TH - 1) * STRIDE + 3, PW = (TW - 1) * STRIDE + 3;   // input patch
  constexpr int PPIX = (PH * PW + 15) / 16 * 16;   // ... rounded to whole swizzle groups
  constexpr int PBLK = (PPIX * CV + 63) / 64;      // 1 KiB load blocks of the patch
  constexpr int PL = (PBLK + NW - 1) / NW;         // ... per wave
  constexpr int PATCH = PL * NW * 64;              // slots (16 bytes) of the patch buffer
  constexpr int APLANE = BM * BKV, ACT = KP * APLANE;   // depthwise output tile: KP planes of [BM][64 B]
  constexpr int WB = BN / 16;                      // 1 KiB load blocks of one filter plane
  static_assert(WB % NW == 0, "filter blocks must divide over the waves");
  constexpr int WL = WB / NW;
  constexpr int FPLANE = BN * BKV, FSTAGE = KP * FPLANE;
  constexpr int EP = WTN / 4 + 1;                  // epilogue staging pitch, as in the implicit-GEMM kernel
  constexpr int MAIN = PATCH + ACT + 2 * FSTAGE, EPI = NW * 32 * EP;
  constexpr int IH = (MH - 1) * STRIDE + 3, IW = (MW - 1) * STRIDE + 3;   // patch of one micro-tile
  constexpr int MTX = TW / MW, MTY = TH / MH;
  constexpr int ITEMS = MTX * MTY * CV;            // (micro-tile, channel vector) work items per chunk
  constexpr int NIT = (ITEMS + NT - 1) / NT;
  static_assert(NT % CV == 0, "a thread keeps one channel vector through all its items");
  constexpr int KSTEPS = KP * (BKV / 2);
  typedef Mma<false>::acc_t acc_t;
  __shared__ uint4 lds[MAIN > EPI ? MAIN : EPI];
  uint4* const patch = lds;
  uint4* const act = lds + PATCH;
  uint4* const filt = lds + PATCH + ACT;

  const ConvArgs& pw = a.pw;
  asm volatile("" ::"s"(a.x), "s"(a.dw_w), "s"(a.dw_bias), "s"(a.dw_scale), "s"(a.dw_shift), "s"(a.dw_flags), "s"(a.N), "s"(a.H),
               "s"(a.W), "s"(a.C), "s"(a.Ho), "s"(a.Wo), "s"(a.tiles_x), "s"(a.tiles_y), "s"(a.tiles_n));
  asm volatile("" ::"s"(pw.w), "s"(pw.y), "s"(pw.bias), "s"(pw.scale), "s"(pw.shift), "s"(pw.K), "s"(pw.Kp), "s"(pw.flags),
               "s"(pw.param_vec));
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  // (image, tile row, tile column, channel tile), channel tile fastest: the workgroups that share a patch are neighbours
  int t = xcd_remap(blockIdx.x, gridDim.x);
  const int tile_n = t % a.tiles_n;
  t /= a.tiles_n;
  const int tx = t % a.tiles_x;
  t /= a.tiles_x;
  const int ty = t % a.tiles_y;
  const int n = t / a.tiles_y;
  const int oy0 = ty * TH, ox0 = tx * TW, n0 = tile_n * BN;
  const int iy0 = oy0 * STRIDE - 1, ix0 = ox0 * STRIDE - 1;   // input coordinates of patch pixel (0, 0)

  // ---- what this lane loads: PL patch vectors and WL filter vectors per 64-byte plane
  unsigned x_off[PL];
#pragma unroll
  for (int j = 0; j < PL; ++j) {
    const int v = ((j * NW + wave) * 64 + lane);
    const int slot = v / CV, cv = v % CV;
    const int p = patch_slot<CV>(slot);
    const int py = p / PW, px = p - py * PW;
    const int iy = iy0 + py, ix = ix0 + px;
    const bool ok = p < PH * PW && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
    x_off[j] = ok ? (unsigned)((((n * a.H + iy) * a.W + ix) * a.C + cv * 8) * 2) : kOob;
  }
  const int srow = lane >> 2, sphys = lane & 3;
  unsigned w_off[WL];
#pragma unroll
  for (int j = 0; j < WL; ++j) {
    const int row = (wave * WL + j) * 16 + srow;
    const int kvl = sphys ^ lds_swizzle(row);
    const int ch = n0 + row;
    w_off[j] = ch < pw.K ? (unsigned)((ch * pw.Kp + kvl * 8) * 2) : kOob;
  }
  const intx4 rs_x = make_rsrc(a.x, (unsigned)a.N * a.H * a.W * a.C * 2u);
  const intx4 rs_w = make_rsrc(pw.w, (unsigned)pw.K * pw.Kp * 2u);
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) uint4*)(&lds[0]);
  auto issue_patch = [&](int kc) {
#pragma unroll
    for (int j = 0; j < PL; ++j)   // (an out-of-range offset plus the chunk position stays out of range)
      lds_dma16(rs_x, lds_base + (unsigned)((j * NW + wave) * 64) * 16u, x_off[j] + (unsigned)(kc * CK * 2));
  };
  auto issue_filters = [&](int kc, int stage) {
#pragma unroll
    for (int plane = 0; plane < KP; ++plane)
#pragma unroll
      for (int j = 0; j < WL; ++j)
        lds_dma16(rs_w, lds_base + (unsigned)(PATCH + ACT + stage * FSTAGE + plane * FPLANE + (wave * WL + j) * 64) * 16u,
                  w_off[j] + (unsigned)((kc * CK + plane * 32) * 2));
  };

  // epilogue constants of the 1x1 conv: their loads leave ahead of everything else
  constexpr int CG = WTN / 8;
  const int ech = n0 + wn * WTN + (lane % CG) * 8;
  RawLaneParams rawp;
  fetch_lane_params<false>(pw, ech, rawp);

  const int nch = a.C / CK;
  issue_patch(0);
  issue_filters(0, 0);

  acc_t acc[TN][TM];
#pragma unroll
  for (int tn = 0; tn < TN; ++tn)
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tn][tm][v] = 0;

  const int cv = tid % CV;   // the channel vector of every item of this thread
  const float relu_lo = (a.dw_flags & F_RELU) ? 0.f : -__builtin_inff();
  const int lrow = lane & 31, lhalf = lane >> 5;

  for (int kc = 0; kc < nch; ++kc) {
    // depthwise filters and constants of this thread's 8 channels in the chunk
    const int c = kc * CK + cv * 8;
    const _Float16* w = static_cast<const _Float16*>(a.dw_w) + c;   // [r][s][c]
    uint4 wv[9];
#pragma unroll
    for (int k = 0; k < 9; ++k) wv[k] = *reinterpret_cast<const uint4*>(w + (long)k * a.C);
    float mul[8], add[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float sc = (a.dw_flags & F_BN) ? a.dw_scale[c + e] : 1.f;
      const float sf = (a.dw_flags & F_BN) ? a.dw_shift[c + e] : 0.f;
      const float b = (a.dw_flags & F_BIAS) ? a.dw_bias[c + e] : 0.f;
      mul[e] = sc;
      add[e] = b * sc + sf;  // (acc + b)*sc + sf
    }
    wait_loads<0>();
    barrier_fenced();   // patch and filters of chunk kc are in LDS; the other filter stage and the tile are free
    if (kc + 1 < nch) issue_filters(kc + 1, (kc + 1) & 1);

    // ---- depthwise: MH x MW outputs x 8 channels per item, patch rows streamed through registers
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int item = it * NT + tid;
      if (NIT * NT != ITEMS && item >= ITEMS) break;
      const int mt = item / CV;
      const int mtx = mt % MTX, mty = mt / MTX;
      const int pbase = (mty * MH * STRIDE) * PW + mtx * MW * STRIDE;
      float dacc[MH][MW][8];
#pragma unroll
      for (int i = 0; i < MH; ++i)
#pragma unroll
        for (int j = 0; j < MW; ++j)
#pragma unroll
          for (int e = 0; e < 8; ++e) dacc[i][j][e] = 0.f;
#pragma unroll
      for (int r = 0; r < IH; ++r) {   // patch row r feeds output row i through filter row fr = r - i*STRIDE
        uint4 xr[IW];
#pragma unroll
        for (int q = 0; q < IW; ++q) xr[q] = patch[patch_slot<CV>(pbase + r * PW + q) * CV + cv];
#pragma unroll
        for (int i = 0; i < MH; ++i) {
          const int fr = r - i * STRIDE;
          if (fr < 0 || fr > 2) continue;
#pragma unroll
          for (int fs = 0; fs < 3; ++fs) {
            const uint4 ww = wv[fr * 3 + fs];
            const unsigned wr[4] = {ww.x, ww.y, ww.z, ww.w};
#pragma unroll
            for (int j = 0; j < MW; ++j) {
              const uint4 xx = xr[j * STRIDE + fs];
              const unsigned xh[4] = {xx.x, xx.y, xx.z, xx.w};
#pragma unroll
              for (int h = 0; h < 4; ++h) {
                fma_mix_lo(dacc[i][j][2 * h], xh[h], wr[h]);
                fma_mix_hi(dacc[i][j][2 * h + 1], xh[h], wr[h]);
              }
            }
          }
        }
      }
#pragma unroll
      for (int i = 0; i < MH; ++i)
#pragma unroll
        for (int j = 0; j < MW; ++j) {
          half8 o;
#pragma unroll
          for (int e = 0; e < 8; ++e) o[e] = (_Float16)fmaxf(dacc[i][j][e] * mul[e] + add[e], relu_lo);
          const int row = (mty * MH + i) * TW + mtx * MW + j;
          act[(cv / BKV) * APLANE + lds_slot(row, cv % BKV)] = __builtin_bit_cast(uint4, o);
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    barrier_fenced();   // the tile is complete, the patch is free
    if (kc + 1 < nch) issue_patch(kc + 1);

    // ---- 1x1 conv over the chunk
    const uint4* fs = filt + (kc & 1) * FSTAGE;
#pragma unroll
    for (int k = 0; k < KSTEPS; ++k) {
      const uint4* xs = act + (k >> 1) * APLANE;
      const uint4* ws = fs + (k >> 1) * FPLANE;
      const int kq = 2 * (k & 1) + lhalf;
      uint4 wf[TN], xf[TM];
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) wf[tn] = ws[lds_slot(wn * WTN + tn * 32 + lrow, kq)];
#pragma unroll
      for (int tm = 0; tm < TM; ++tm) xf[tm] = xs[lds_slot(wm * WTM + tm * 32 + lrow, kq)];
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = Mma<false>::mma(wf[tn], xf[tm], acc[tn][tm]);
    }
  }

  // ---- epilogue of the 1x1 conv: transposition through LDS, then 8 consecutive channels of one pixel per lane
  LaneParams lp;
  finish_lane_params<false>(rawp, lp);
  wait_loads<0>();
  barrier_fenced();   // every wave is done with the tile and the ring
  uint4* stg = lds + wave * (32 * EP);
  constexpr int PPI = 64 / CG;
  const int epix = lane / CG, ecg = lane % CG;
  const bool vec_ok = (pw.K & 7) == 0;
  const OutLoc ol{nullptr, 0, 0, 0};
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint4 v;
        v.x = as_u32(acc[tn][tm][4 * g]);
        v.y = as_u32(acc[tn][tm][4 * g + 1]);
        v.z = as_u32(acc[tn][tm][4 * g + 2]);
        v.w = as_u32(acc[tn][tm][4 * g + 3]);
        stg[lrow * EP + tn * 8 + 2 * g + lhalf] = v;
      }
#pragma unroll
    for (int it = 0; it < 32 / PPI; ++it) {
      const int pix = it * PPI + epix;
      const uint4 lo = stg[pix * EP + ecg * 2], hi = stg[pix * EP + ecg * 2 + 1];
      const unsigned raw[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      const int row = wm * WTM + tm * 32 + pix;   // row of the tile = (row / TW, row % TW) of the rectangle
      const int ry = row / TW, rx = row - ry * TW;
      const int oy = oy0 + ry, ox = ox0 + rx;
      if (row >= TH * TW || oy >= a.Ho || ox >= a.Wo || ech >= pw.K) continue;
      const int m = (n * a.Ho + oy) * a.Wo + ox;
      finish_store8<false, false, false>(pw, raw, m, ech, lp, ol, vec_ok);
    }
  }
}

struct DwPwVariant {
  int stride, th, tw, mh, mw, waves_m, waves_n, tm, tn, kp;
  constexpr int bn() const { return waves_n * tn * 32; }
  constexpr int ck() const { return kp * 32; }
};
// must match launch_variant
constexpr DwPwVariant kVariants[] = {
    {1, 8, 16, 1, 2, 2, 2, 2, 1, 1},   // 0: 8 x 16 pixels x 64 channels, 32-channel chunks (the widest images)
    {1, 4, 28, 1, 4, 2, 2, 2, 2, 1},   // 1: 4 x 28 x 128
    {1, 4, 28, 2, 4, 2, 2, 2, 2, 2},   // 2: 4 x 28 x 128, 64-channel chunks
    {1, 8, 14, 2, 2, 2, 2, 2, 2, 2},   // 3: 8 x 14 x 128
    {1, 4, 14, 1, 2, 2, 2, 1, 2, 2},   // 4: 4 x 14 x 128 in a 64-row tile
    {1, 7, 7, 1, 1, 2, 2, 1, 2, 2},    // 5: a whole 7 x 7 image x 128
    {2, 4, 28, 1, 2, 2, 2, 2, 2, 1},   // 6: stride 2, 4 x 28 x 128
    {2, 4, 14, 1, 2, 2, 2, 1, 2, 1},   // 7: stride 2, 4 x 14 x 128 in a 64-row tile
    {2, 7, 7, 1, 1, 2, 2, 1, 2, 1},    // 8: stride 2, 7 x 7 x 128
    {2, 8, 14, 1, 2, 2, 2, 2, 2, 1},   // 9: stride 2, 8 x 14 x 128
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

template <int STRIDE, int TH, int TW, int MH, int MW, int WAVES_M, int WAVES_N, int TM, int TN, int KP>
hipError_t launch_one(const DwPwArgs& a, hipStream_t st) {
  DwPwArgs b = a;
  b.tiles_x = (a.Wo + TW - 1) / TW;
  b.tiles_y = (a.Ho + TH - 1) / TH;
  b.tiles_n = (a.pw.K + WAVES_N * TN * 32 - 1) / (WAVES_N * TN * 32);
  const long wgs = (long)a.N * b.tiles_y * b.tiles_x * b.tiles_n;
  hipLaunchKernelGGL((dwpw_fused_kernel<STRIDE, TH, TW, MH, MW, WAVES_M, WAVES_N, TM, TN, KP>), dim3((unsigned)wgs),
                     dim3(64 * WAVES_M * WAVES_N), 0, st, b);
  return hipGetLastError();
}

hipError_t launch_variant(const DwPwArgs& a, int v, hipStream_t st) {
  switch (v) {
    case 0: return launch_one<1, 8, 16, 1, 2, 2, 2, 2, 1, 1>(a, st);
    case 1: return launch_one<1, 4, 28, 1, 4, 2, 2, 2, 2, 1>(a, st);
    case 2: return launch_one<1, 4, 28, 2, 4, 2, 2, 2, 2, 2>(a, st);
    case 3: return launch_one<1, 8, 14, 2, 2, 2, 2, 2, 2, 2>(a, st);
    case 4: return launch_one<1, 4, 14, 1, 2, 2, 2, 1, 2, 2>(a, st);
    case 5: return launch_one<1, 7, 7, 1, 1, 2, 2, 1, 2, 2>(a, st);
    case 6: return launch_one<2, 4, 28, 1, 2, 2, 2, 2, 2, 1>(a, st);
    case 7: return launch_one<2, 4, 14, 1, 2, 2, 2, 1, 2, 1>(a, st);
    case 8: return launch_one<2, 7, 7, 1, 1, 2, 2, 1, 2, 1>(a, st);
    default: return launch_one<2, 8, 14, 1, 2, 2, 2, 2, 2, 1>(a, st);
  }
}

}  // namespace

int dwpw_variant_count() { return kNumVariants; }

bool dwpw_supported(const DwPwArgs& a, int v) {
  if (v < 0 || v >= kNumVariants) return false;
  const DwPwVariant& t = kVariants[v];
  const size_t lim = 0x7fffffffu;   // 32-bit buffer offsets, 2^31 marks "out of range"
  return t.stride == a.stride && a.C % t.ck() == 0 && (a.pw.K & 7) == 0 && (size_t)a.N * a.H * a.W * a.C * 2 <= lim &&
         (size_t)a.pw.K * a.pw.Kp * 2 <= lim;
}

// The variant whose rectangle wastes the fewest rows on this image, the longer chunks where the
// channel count allows; -1: no variant takes the shape.
int dwpw_pick(const DwPwArgs& a) {
  int best = -1;
  double best_cost = 0;
  for (int v = 0; v < kNumVariants; ++v) {
    if (!dwpw_supported(a, v)) continue;
    const DwPwVariant& t = kVariants[v];
    const long tiles = (long)((a.Ho + t.th - 1) / t.th) * ((a.Wo + t.tw - 1) / t.tw);
    const int bm = t.waves_m * t.tm * 32;
    // rows computed per useful row, a little in favour of long chunks and wide channel tiles
    double cost = (double)tiles * bm / ((double)a.Ho * a.Wo);
    if (t.kp == 1) cost *= 1.05;
    if (t.bn() < a.pw.K && t.bn() < 128) cost *= 1.5;
    if (best < 0 || cost < best_cost) {
      best = v;
      best_cost = cost;
    }
  }
  return best;
}

hipError_t launch_dwpw(const DwPwArgs& a, int variant, hipStream_t st) { return launch_variant(a, variant, st); }

void dwpw_kernel_name(int variant, char* buf, size_t len) {
  const DwPwVariant& t = kVariants[variant];
  snprintf(buf, len, "dwpw_fused_kernel<%d, %d, %d, %d, %d, %d, %d, %d, %d, %d>", t.stride, t.th, t.tw, t.mh, t.mw, t.waves_m,
           t.waves_n, t.tm, t.tn, t.kp);
}

}  // namespace relay
