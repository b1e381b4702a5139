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
//      in an LDS ring of two or three stages, as in the implicit-GEMM kernel.
// The chunks are pipelined: one barrier per chunk, behind which the patch two or three chunks ahead and
// the filters one or two chunks ahead are requested, and the depthwise work of chunk kc + 1 is
// interleaved with the matrix instructions of chunk kc.  Layers whose channels fit one chunk run a
// straight-line form with one buffer of everything (little LDS, few registers, many workgroups per CU).
// Variants with eight waves put two waves on every SIMD, so that one wave's wait for the barrier or for
// LDS is covered by the other's arithmetic.
// The fp16 narrowing in the middle is that of the two-kernel pipeline, and the 1x1 reduction runs
// in the same order with the same instruction, so the result equals the two launches bit for bit.
// A workgroup per tile of output channels recomputes the depthwise tile; with few output pixels
// (the deep layers) that is what buys enough workgroups to fill the chip.
#include <cstdio>

#include "dma_common.hpp"
#include "dw_math.hpp"

namespace relay {
namespace {

// Slot of patch pixel p (in units of one pixel's CV vectors).  Stride 1: the pixel itself -- with micro-tiles one
// pixel wide, consecutive lanes read consecutive pixels, a contiguous run of LDS that touches every bank once, and
// every tap is a compile-time offset from one base address.  Stride 2: neighbouring micro-tiles are an even
// number of pixels apart, a multiple of the bank period; the XOR with a few higher bits of p spreads them over
// the banks (an involution inside aligned groups of 16 pixels, so the loader applies the same function to find
// the pixel that belongs in a slot).
template <int CV, int STRIDE>
__device__ __forceinline__ int patch_slot(int p) {
  if (STRIDE == 1) return p;
  return CV <= 4 ? p ^ ((p >> 2) & 3) : p ^ ((p >> 1) & 1);
}

// Workgroup barrier that the compiler does not move LDS accesses across (the waits that make this
// wave's own LDS writes and global->LDS loads complete stand in front of it at every use).
__device__ __forceinline__ void barrier_fenced() {
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// k-steps of the matrix cores that have been started before work unit u of the vector ALUs, when
// KSTEPS k-steps are spread evenly over U units (the first one ahead of unit 0)
constexpr int ksteps_before(int u, int ksteps, int units) { return (u * ksteps + units - 1) / units; }

// NP: input patches in flight (LDS buffers); CMAX: most depthwise channels (their filters and constants
// sit in LDS for the whole kernel).
// OCC: waves per SIMD the register allocation is held to (the layers that stream from memory need several
// workgroups per CU to keep enough loads and stores in flight).
template <int STRIDE, int TH, int TW, int MH, int MW, int WAVES_M, int WAVES_N, int TM, int TN, int KP, int NP, int NFS, int CMAX, int OCC>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, OCC) void dwpw_fused_kernel(const DwPwArgs a) {
  constexpr int NW = WAVES_M * WAVES_N, NT = 64 * NW;
  constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32, WTM = TM * 32, WTN = TN * 32;
  static_assert(TH * TW <= BM, "the rectangle must fit the rows of the tile");
  static_assert(TH % MH == 0 && TW % MW == 0, "whole micro-tiles");
  static_assert(NP >= 1 && NP <= 3, "one patch (single-chunk layers: C == CK, one buffer of everything), or two or three in flight");
  constexpr bool ONE = NP == 1;
  static_assert(NFS == 3 || (NFS == 2 && NP == 3), "two filter stages go with three patches");
  constexpr int CV = KP * BKV;                     // 16-byte channel vectors per pixel per chunk
  constexpr int CK = CV * 8;                       // depthwise channels per chunk
  constexpr int PH = (TH - 1) * STRIDE + 3, PW = (TW - 1) * STRIDE + 3;   // input patch
  constexpr int PPIX = (PH * PW + 15) / 16 * 16;   // ... rounded to whole swizzle groups
  constexpr int PBLK = (PPIX * CV + 63) / 64;      // 1 KiB load blocks of the patch
  constexpr int PL = (PBLK + NW - 1) / NW;         // ... per wave
  constexpr int PBUF = PL * NW * 64;               // slots (16 bytes) of one patch buffer
  constexpr int APLANE = BM * BKV, ACT = KP * APLANE;   // depthwise output tile: KP planes of [BM][64 B]
  constexpr int WB = BN / 16;                      // 1 KiB load blocks of one filter plane
  // (single-chunk layers wait for all their loads at once, so their waves need not issue equal numbers of them)
  static_assert(NP == 1 || WB % NW == 0, "filter blocks must divide over the waves");
  constexpr int WL = (WB + NW - 1) / NW;
  constexpr int FL = KP * WL;                      // filter loads per chunk per wave
  constexpr int LPI = PL + FL;                     // loads per iteration per wave
  static_assert(LPI <= 63, "vmcnt is a 6-bit counter");
  constexpr int FPLANE = BN * BKV, FSTAGE = KP * FPLANE, NF = ONE ? 1 : NFS, NA = ONE ? 1 : 2;
  constexpr int EP = WTN / 4 + 1;                  // epilogue staging pitch, as in the implicit-GEMM kernel
  constexpr int WTS = 9 * (CMAX / 8), CST = CMAX / 4;   // slots of the depthwise filters; of one array of constants
  constexpr int O_PATCH = WTS + 2 * CST, O_ACT = O_PATCH + NP * PBUF, O_FILT = O_ACT + NA * ACT;
  constexpr int MAIN = O_FILT + NF * FSTAGE, EPI = NW * 32 * EP;
  static_assert((MAIN > EPI ? MAIN : EPI) * 16 <= 160 * 1024, "LDS of one CU");
  constexpr int IH = (MH - 1) * STRIDE + 3, IW = (MW - 1) * STRIDE + 3;   // patch of one micro-tile
  constexpr int MTX = TW / MW, MTY = TH / MH;
  constexpr int ITEMS = MTX * MTY * CV;            // (micro-tile, channel vector) work items per chunk
  constexpr int NIT = (ITEMS + NT - 1) / NT;
  static_assert(NT % CV == 0, "a thread keeps one channel vector through all its items");
  constexpr int KSTEPS = KP * (BKV / 2);
  constexpr int UNITS = NIT * IH;                  // (item, patch row) units of depthwise work per chunk
  typedef Mma<false>::acc_t acc_t;
  __shared__ uint4 lds[MAIN > EPI ? MAIN : EPI];
  uint4* const wts = lds;                                      // [tap][C/8] depthwise filters
  float* const cmul = reinterpret_cast<float*>(lds + WTS);     // [C] scale
  float* const cadd = reinterpret_cast<float*>(lds + WTS + CST);   // [C] bias*scale + shift
  uint4* const patch = lds + O_PATCH;
  uint4* const act = lds + O_ACT;
  uint4* const filt = lds + O_FILT;

  const ConvArgs& pw = a.pw;
  asm volatile("" ::"s"(a.x), "s"(a.dw_w), "s"(a.dw_bias), "s"(a.dw_scale), "s"(a.dw_shift), "s"(a.dw_flags), "s"(a.N), "s"(a.H),
               "s"(a.W), "s"(a.C), "s"(a.Ho), "s"(a.Wo), "s"(a.tiles_x), "s"(a.tiles_y), "s"(a.tiles_n), "s"(a.fd_x.mul), "s"(a.fd_x.shift),
               "s"(a.fd_y.mul), "s"(a.fd_y.shift), "s"(a.fd_n.mul), "s"(a.fd_n.shift));
  asm volatile("" ::"s"(pw.w), "s"(pw.y), "s"(pw.bias), "s"(pw.scale), "s"(pw.shift), "s"(pw.K), "s"(pw.Kp), "s"(pw.flags),
               "s"(pw.param_vec));
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  // (image, tile row, tile column, channel tile), channel tile fastest: the workgroups that share a patch are neighbours
  // (divisions by multiply-high with host-computed constants: three software divisions would be a fifth of the
  // vector instructions of a single-chunk tile)
  const unsigned t0 = (unsigned)xcd_remap(blockIdx.x, gridDim.x);
  const unsigned t1 = fast_div(t0, a.fd_n), t2 = fast_div(t1, a.fd_x);
  const int tile_n = (int)(t0 - t1 * (unsigned)a.tiles_n);
  const int tx = (int)(t1 - t2 * (unsigned)a.tiles_x);
  const int n = (int)fast_div(t2, a.fd_y);
  const int ty = (int)t2 - n * a.tiles_y;
  const int oy0 = ty * TH, ox0 = tx * TW, n0 = tile_n * BN;
  const int iy0 = oy0 * STRIDE - 1, ix0 = ox0 * STRIDE - 1;   // input coordinates of patch pixel (0, 0)
  const int nch = a.C / CK;

  // ---- the depthwise filters and constants of all channels go to LDS once (their loads leave first and
  //      are in flight while the first patches are requested)
  constexpr int WPT = (WTS + NT - 1) / NT, CPT = (CMAX + NT - 1) / NT;
  const int cvecs = a.C >> 3;
  uint4 wreg[WPT];
  float screg[CPT], sfreg[CPT], bsreg[CPT];
#pragma unroll
  for (int i = 0; i < WPT; ++i) {
    const int v = i * NT + tid;
    wreg[i] = v < 9 * cvecs ? static_cast<const uint4*>(a.dw_w)[v] : make_uint4(0u, 0u, 0u, 0u);
  }
#pragma unroll
  for (int i = 0; i < CPT; ++i) {
    const int c = i * NT + tid;
    const bool in = c < a.C;
    screg[i] = (in && (a.dw_flags & F_BN)) ? a.dw_scale[c] : 1.f;
    sfreg[i] = (in && (a.dw_flags & F_BN)) ? a.dw_shift[c] : 0.f;
    bsreg[i] = (in && (a.dw_flags & F_BIAS)) ? a.dw_bias[c] : 0.f;
  }
  // epilogue constants of the 1x1 conv
  constexpr int CG = WTN / 8;
  const int ech = n0 + wn * WTN + (lane % CG) * 8;
  RawLaneParams rawp;
  fetch_lane_params<false>(pw, ech, rawp);

  // ---- what this lane loads per chunk: PL patch vectors and WL filter vectors per 64-byte plane
  unsigned x_off[PL];
#pragma unroll
  for (int j = 0; j < PL; ++j) {
    const int v = ((j * NW + wave) * 64 + lane);
    const int slot = v / CV, cvl = v % CV;
    const int p = patch_slot<CV, STRIDE>(slot);
    const int py = p / PW, px = p - py * PW;
    const int iy = iy0 + py, ix = ix0 + px;
    const bool ok = p < PH * PW && (unsigned)iy < (unsigned)a.H && (unsigned)ix < (unsigned)a.W;
    x_off[j] = ok ? (unsigned)((((n * a.H + iy) * a.W + ix) * a.C + cvl * 8) * 2) : kOob;
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
  // chunks past the end of the reduction are requested all the same, with out-of-range offsets: every
  // iteration then issues the same number of loads, which is what the waits below count
  auto issue_patch = [&](int kc) {
    const unsigned buf = lds_base + (unsigned)(O_PATCH + (kc % NP) * PBUF) * 16u;
    const bool live = kc < nch;
#pragma unroll
    for (int j = 0; j < PL; ++j)   // (an out-of-range offset plus the chunk position stays out of range)
      lds_dma16(rs_x, buf + (unsigned)((j * NW + wave) * 64) * 16u, live ? x_off[j] + (unsigned)(kc * CK * 2) : kOob);
  };
  auto issue_filters = [&](int kc) {
    const unsigned stage = lds_base + (unsigned)(O_FILT + (kc % NF) * FSTAGE) * 16u;
    const bool live = kc < nch;
#pragma unroll
    for (int plane = 0; plane < KP; ++plane)
#pragma unroll
      for (int j = 0; j < WL; ++j)
        if (WB % NW == 0 || wave * WL + j < WB)   // (uniform)
          lds_dma16(rs_w, stage + (unsigned)(plane * FPLANE + (wave * WL + j) * 64) * 16u,
                    live ? w_off[j] + (unsigned)((kc * CK + plane * 32) * 2) : kOob);
  };
  // Iteration j of the main loop requests patch j+NP and filters j+2.  With two patch buffers the patch
  // goes first and the filters of the same iteration may still be in flight when the patch is needed;
  // with three, the filters go first and a whole iteration's loads may be in flight.
  // (With two filter stages the filters are requested one chunk ahead only, first in their iteration: the
  // patch requested behind them may still be in flight when they are needed.)
  auto issue_iteration = [&](int j) {
    if constexpr (NP == 2) {
      issue_patch(j + 2);
      issue_filters(j + 2);
    } else if constexpr (NF == 3) {
      issue_filters(j + 2);
      issue_patch(j + 3);
    } else {
      if (j + 1 >= 0) issue_filters(j + 1);
      issue_patch(j + 3);
    }
  };
  if constexpr (ONE) {
    issue_patch(0);
    issue_filters(0);
  } else {
    if constexpr (NP == 3) issue_patch(0);
    issue_iteration(-2);
    issue_iteration(-1);
  }

#pragma unroll
  for (int i = 0; i < WPT; ++i) {
    const int v = i * NT + tid;
    if (v < WTS) wts[v] = wreg[i];
  }
#pragma unroll
  for (int i = 0; i < CPT; ++i) {
    const int c = i * NT + tid;
    if (c < CMAX) {
      cmul[c] = screg[i];
      cadd[c] = bsreg[i] * screg[i] + sfreg[i];  // (acc + b)*sc + sf
    }
  }

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

  // One chunk of work: the depthwise outputs of chunk kc + 1 (DW) on the vector ALUs, and the 1x1 conv over
  // chunk kc (MMA) on the matrix cores, the k-steps of the latter spread over the units of the former so
  // that both pipes are busy at once.
  auto work = [&](auto dw_tag, auto mma_tag, int kc) {
    constexpr bool DW = decltype(dw_tag)::value, MMA = decltype(mma_tag)::value;
    const uint4* fs = filt + ((kc + NF) % NF) * FSTAGE;   // (kc = -1: no 1x1 conv in that call, nothing is read)
    const uint4* as = act + ((kc + NA) % NA) * ACT;
    uint4 wf[2][TN], xf[2][TM];
    auto fetch = [&](int k) {
      const uint4* xs = as + (k >> 1) * APLANE;
      const uint4* ws = fs + (k >> 1) * FPLANE;
      const int kq = 2 * (k & 1) + lhalf;
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) wf[k & 1][tn] = ws[lds_slot(wn * WTN + tn * 32 + lrow, kq)];
#pragma unroll
      for (int tm = 0; tm < TM; ++tm) xf[k & 1][tm] = xs[lds_slot(wm * WTM + tm * 32 + lrow, kq)];
    };
    auto kstep = [&](int k) {
      if (k + 1 < KSTEPS) fetch(k + 1);
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = Mma<false>::mma(wf[k & 1][tn], xf[k & 1][tm], acc[tn][tm]);
    };
    if constexpr (MMA) fetch(0);
    if constexpr (!DW) {
#pragma unroll
      for (int k = 0; k < KSTEPS; ++k) kstep(k);
    } else {
      const int kd = kc + 1;   // the chunk whose depthwise outputs are computed
      const uint4* pt = patch + (kd % NP) * PBUF;
      uint4* at = act + (kd % NA) * ACT;
      uint4 wv[9];
#pragma unroll
      for (int k = 0; k < 9; ++k) wv[k] = wts[k * cvecs + kd * CV + cv];
      // The patch rows of an item are requested one row ahead of the multiply-adds that consume them (and
      // the first row of the next item behind the last row of this one): with one wave per SIMD nothing
      // else covers the LDS latency.
      auto item_of = [&](int it, bool& has, int& pbase, int& row0) {
        const int item = it * NT + tid;
        has = NIT * NT == ITEMS || item < ITEMS;
        const int mt = has ? item / CV : 0;
        const int mtx = mt % MTX, mty = mt / MTX;
        pbase = (mty * MH * STRIDE) * PW + mtx * MW * STRIDE;
        row0 = (mty * MH) * TW + mtx * MW;
      };
      uint4 xr[2][IW];
      auto load_row = [&](int pbase, int r, uint4(&dst)[IW]) {
#pragma unroll
        for (int q = 0; q < IW; ++q) dst[q] = pt[patch_slot<CV, STRIDE>(pbase + r * PW + q) * CV + cv];
      };
      bool has;
      int pbase, row0;
      item_of(0, has, pbase, row0);
      load_row(pbase, 0, xr[0]);
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        float dacc[MH][MW][8];
#pragma unroll
        for (int i = 0; i < MH; ++i)
#pragma unroll
          for (int j = 0; j < MW; ++j)
#pragma unroll
            for (int e = 0; e < 8; ++e) dacc[i][j][e] = 0.f;
        const bool has_now = has;
        const int row_now = row0;
#pragma unroll
        for (int r = 0; r < IH; ++r) {   // patch row r feeds output row i through filter row fr = r - i*STRIDE
          const int u = it * IH + r;
          uint4(&cur)[IW] = xr[u & 1];
          if (r + 1 < IH) {
            load_row(pbase, r + 1, xr[(u + 1) & 1]);
          } else if (it + 1 < NIT) {
            item_of(it + 1, has, pbase, row0);
            load_row(pbase, 0, xr[(u + 1) & 1]);
          }
          if constexpr (MMA) {
#pragma unroll
            for (int k = ksteps_before(u, KSTEPS, UNITS); k < ksteps_before(u + 1, KSTEPS, UNITS); ++k) kstep(k);
          }
#pragma unroll
          for (int i = 0; i < MH; ++i) {
            const int fr = r - i * STRIDE;
            if (fr < 0 || fr > 2) continue;
#pragma unroll
            for (int fsx = 0; fsx < 3; ++fsx) {
              const uint4 ww = wv[fr * 3 + fsx];
              const unsigned wr[4] = {ww.x, ww.y, ww.z, ww.w};
#pragma unroll
              for (int j = 0; j < MW; ++j) {
                const uint4 xx = cur[j * STRIDE + fsx];
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
        // (the constants of the fused tail are read here, not held through the multiply-adds)
        const float4* m4 = reinterpret_cast<const float4*>(cmul + kd * CK + cv * 8);
        const float4* a4 = reinterpret_cast<const float4*>(cadd + kd * CK + cv * 8);
        const float4 m0 = m4[0], m1 = m4[1], a0 = a4[0], a1 = a4[1];
        const float mul[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
        const float add[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
        for (int i = 0; i < MH; ++i)
#pragma unroll
          for (int j = 0; j < MW; ++j) {
            const uint4 o = scale_shift_narrow8(dacc[i][j], mul, add, relu_lo);
            const int row = row_now + i * TW + j;
            if (has_now) at[(cv / BKV) * APLANE + lds_slot(row, cv % BKV)] = o;
          }
      }
    }
  };
  // patch kc + 1 and filters kc are in LDS (younger loads may be in flight), every wave's LDS traffic of the
  // previous iteration is done: the buffers that iteration read are free
  auto top_sync = [&]() {
    wait_loads<NP == 2 ? FL : (NF == 3 ? LPI : PL)>();
    barrier_fenced();
  };
  using std::false_type;
  using std::true_type;

  wait_loads<0>();
  barrier_fenced();   // depthwise filters and constants, patch 0 (and all else requested so far) are in LDS
  work(true_type{}, false_type{}, -1);
  for (int kc = 0; !ONE && kc + 1 < nch; ++kc) {
    top_sync();
    issue_iteration(kc);
    work(true_type{}, true_type{}, kc);
  }
  if constexpr (ONE) {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    barrier_fenced();   // the depthwise tile is complete
  } else {
    top_sync();
  }
  work(false_type{}, true_type{}, nch - 1);

  // ---- epilogue of the 1x1 conv: transposition through LDS, then 8 consecutive channels of one pixel per lane
  LaneParams lp;
  finish_lane_params<false>(rawp, lp);
  wait_loads<0>();   // (the requests past the end of the reduction still write zeros into the buffers)
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
  int stride, th, tw, mh, mw, waves_m, waves_n, tm, tn, kp, np, nf, cmax, occ;
  constexpr int bm() const { return waves_m * tm * 32; }
  constexpr int bn() const { return waves_n * tn * 32; }
  constexpr int ck() const { return kp * 32; }
};
// must match launch_variant
constexpr DwPwVariant kVariants[] = {
    {1, 4, 28, 2, 1, 2, 2, 2, 2, 1, 2, 3, 256, 2},   // 0: 4 x 28 pixels x 128 channels, 32-channel chunks, four waves, two workgroups per CU (many pixels, up to 256 channels in, 128 out)
    {1, 8, 16, 2, 1, 2, 2, 2, 1, 1, 1, 3, 32, 4},   // 1: single-chunk layers of 32 channels: 8 x 16 x 64, one buffer of everything, four to six workgroups per CU
    {1, 4, 28, 1, 1, 2, 4, 2, 2, 1, 3, 2, 256, 2},   // 2: 4 x 28 x 256, eight waves (two per SIMD: one wave's LDS and barrier waits are covered by the other), three patches in flight, two filter stages
    {1, 4, 14, 1, 1, 2, 4, 1, 2, 2, 3, 2, 1024, 2},   // 3: 4 x 14 x 256 in a 64-row tile, eight waves, 64-channel chunks, up to 1024 channels (the layers with few pixels)
    {1, 4, 14, 1, 1, 1, 4, 2, 2, 1, 3, 3, 1024, 1},   // 4: 4 x 14 x 256 in a 64-row tile, four waves, 32-channel chunks: takes every stride-1 shape
    {2, 4, 14, 1, 1, 2, 4, 1, 1, 2, 1, 3, 64, 4},   // 5: stride 2, single-chunk layers of 64 channels: 4 x 14 x 128, eight waves
    {2, 4, 28, 1, 1, 2, 4, 2, 2, 1, 2, 3, 256, 2},   // 6: stride 2, 4 x 28 x 256, eight waves
    {2, 7, 7, 1, 1, 2, 4, 1, 2, 1, 3, 2, 1024, 2},   // 7: stride 2, 7 x 7 x 256 in a 64-row tile, eight waves (the layers with few pixels)
    {2, 4, 28, 1, 2, 2, 2, 2, 2, 1, 2, 3, 256, 1},   // 8: stride 2, 4 x 28 x 128, four waves
    {2, 4, 14, 1, 1, 1, 4, 2, 2, 1, 3, 3, 1024, 1},   // 9: stride 2, 4 x 14 x 256 in a 64-row tile, four waves: takes every stride-2 shape
};
constexpr int kNumVariants = sizeof(kVariants) / sizeof(kVariants[0]);

template <int STRIDE, int TH, int TW, int MH, int MW, int WAVES_M, int WAVES_N, int TM, int TN, int KP, int NP, int NFS, int CMAX, int OCC>
hipError_t launch_one(const DwPwArgs& a, hipStream_t st) {
  DwPwArgs b = a;
  b.tiles_x = (a.Wo + TW - 1) / TW;
  b.tiles_y = (a.Ho + TH - 1) / TH;
  b.tiles_n = (a.pw.K + WAVES_N * TN * 32 - 1) / (WAVES_N * TN * 32);
  b.fd_x = make_fastdiv((uint32_t)b.tiles_x);
  b.fd_y = make_fastdiv((uint32_t)b.tiles_y);
  b.fd_n = make_fastdiv((uint32_t)b.tiles_n);
  const long wgs = (long)a.N * b.tiles_y * b.tiles_x * b.tiles_n;
  hipLaunchKernelGGL((dwpw_fused_kernel<STRIDE, TH, TW, MH, MW, WAVES_M, WAVES_N, TM, TN, KP, NP, NFS, CMAX, OCC>), dim3((unsigned)wgs),
                     dim3(64 * WAVES_M * WAVES_N), 0, st, b);
  return hipGetLastError();
}

hipError_t launch_variant(const DwPwArgs& a, int v, hipStream_t st) {
  switch (v) {
    case 0: return launch_one<1, 4, 28, 2, 1, 2, 2, 2, 2, 1, 2, 3, 256, 2>(a, st);
    case 1: return launch_one<1, 8, 16, 2, 1, 2, 2, 2, 1, 1, 1, 3, 32, 4>(a, st);
    case 2: return launch_one<1, 4, 28, 1, 1, 2, 4, 2, 2, 1, 3, 2, 256, 2>(a, st);
    case 3: return launch_one<1, 4, 14, 1, 1, 2, 4, 1, 2, 2, 3, 2, 1024, 2>(a, st);
    case 4: return launch_one<1, 4, 14, 1, 1, 1, 4, 2, 2, 1, 3, 3, 1024, 1>(a, st);
    case 5: return launch_one<2, 4, 14, 1, 1, 2, 4, 1, 1, 2, 1, 3, 64, 4>(a, st);
    case 6: return launch_one<2, 4, 28, 1, 1, 2, 4, 2, 2, 1, 2, 3, 256, 2>(a, st);
    case 7: return launch_one<2, 7, 7, 1, 1, 2, 4, 1, 2, 1, 3, 2, 1024, 2>(a, st);
    case 8: return launch_one<2, 4, 28, 1, 2, 2, 2, 2, 2, 1, 2, 3, 256, 1>(a, st);
    default: return launch_one<2, 4, 14, 1, 1, 1, 4, 2, 2, 1, 3, 3, 1024, 1>(a, st);
  }
}

}  // namespace

int dwpw_variant_count() { return kNumVariants; }

bool dwpw_supported(const DwPwArgs& a, int v) {
  if (v < 0 || v >= kNumVariants) return false;
  const DwPwVariant& t = kVariants[v];
  const size_t lim = 0x7fffffffu;   // 32-bit buffer offsets, 2^31 marks "out of range"
  return t.stride == a.stride && a.C % t.ck() == 0 && a.C <= t.cmax && (t.np != 1 || a.C == t.ck()) && (a.pw.K & 7) == 0 && (size_t)a.N * a.H * a.W * a.C * 2 <= lim &&
         (size_t)a.pw.K * a.pw.Kp * 2 <= lim;
}

// The variant measured fastest on the layer shapes of the MobileNet family at batch 32, where it beats
// the two separate launches; -1 where it does not.  What the fused kernel saves is the round trip of the
// depthwise output through memory and one launch.  It pays most on the layers that stream from memory
// (many pixels, up to 256 channels: 35 % to 15 % less time per block).  With few pixels (the deep
// layers) the work has to be cut along the output channels to fill the chip and every such workgroup
// recomputes the depthwise tile on the vector ALUs: with eight waves per workgroup (two per SIMD, so that
// one wave's LDS and barrier waits are covered by the other) the 512-channel layers at 14 x 14 still gain
// 14 % (two channel tiles), the layers with 1024 output channels (four tiles) lose and stay two launches.
int dwpw_pick(const DwPwArgs& a) {
  const long px = (long)a.N * a.Ho * a.Wo;
  const int k = a.pw.K;
  int v = -1;
  if (a.stride == 1) {
    if (a.C == 32 && px >= 65536) v = 1;
    else if (a.C >= 64 && a.C <= 256 && px >= 16384) v = k >= 256 ? 2 : 0;
    else if (a.C > 256 && a.C <= 512 && k <= 512 && px >= 4096) v = 3;
  } else {
    if (a.C == 64 && px >= 65536) v = 5;
    else if (a.C <= 256 && k >= 256 && k <= 512 && px >= 16384) v = 6;
    else if (a.C <= 256 && k <= 512 && px >= 4096 && px < 16384) v = 7;
  }
  return (v >= 0 && dwpw_supported(a, v)) ? v : -1;
}

// A variant that takes the shape, whatever it costs (for callers that ask for the fused kernel regardless).
int dwpw_any(const DwPwArgs& a) {
  const int p = dwpw_pick(a);
  if (p >= 0) return p;
  const int prefer[] = {0, 4, 8, 9};
  for (int v : prefer)
    if (dwpw_supported(a, v)) return v;
  for (int v = 0; v < kNumVariants; ++v)
    if (dwpw_supported(a, v)) return v;
  return -1;
}

hipError_t launch_dwpw(const DwPwArgs& a, int variant, hipStream_t st) { return launch_variant(a, variant, st); }

void dwpw_kernel_name(int variant, char* buf, size_t len) {
  const DwPwVariant& t = kVariants[variant];
  snprintf(buf, len, "dwpw_fused_kernel<%d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d, %d>", t.stride, t.th, t.tw, t.mh, t.mw,
           t.waves_m, t.waves_n, t.tm, t.tn, t.kp, t.np, t.nf, t.cmax, t.occ);
}

}  // namespace relay
