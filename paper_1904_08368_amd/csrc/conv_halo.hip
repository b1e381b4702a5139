// 3x3 / stride 1 / pad 1 conv2d for gfx950 that stages the activations ONCE per channel chunk
// (paper Section 4.1 / 4.2: same fused primitive function as conv_igemm_dma.hip, other schedule).
//
// The implicit-GEMM kernel re-fetches the activation tile for each of the nine filter taps: its
// L2->LDS traffic is what bounds the 3x3 layers of the workloads.  Here the pixels are numbered in
// a "padded-flat" coordinate in which a filter tap is a constant shift:
//     o = n*F + p*P + q,   P = W + 1,  F = (H + 1)*P
// (one shared zero column between image rows, one shared zero row between images: the left
// padding of a row is the right padding of the row before it).  Output position o reads input
// position o + r*P + s for tap (r, s), where input position g holds pixel (row - 1, col - 1) of
// image g / F with (row, col) = divmod(g % F, P), and zero when row == 0 or col == 0.  A
// workgroup owns BM consecutive positions (positions with q == W or p == H are computed and
// dropped: 3-15 % of the work on these images) x BN channels.  Per chunk of CK input channels it
// needs the BM + 2P + 2 input positions from its first one on -- the halo -- which it loads once
// into LDS with global->LDS loads (zero fill by out-of-range offset, as in the other kernel);
// the nine taps then read the same buffer at row offsets r*P + s.  The LDS swizzle is keyed on
// row >> 2 and any 16 consecutive rows cover all banks, so the shifted reads stay conflict-free.
// Filters go through a 3-stage ring, one tap x chunk per stage, exactly as before.
//
// Pipeline: a "step" is one (chunk, tap).  Behind the MFMAs of step i a wave issues the filter
// loads of step i+2 and its share of the NEXT chunk's halo (spread over the first 8 taps, so the
// halo has landed two steps before its chunk starts).  Every step issues the same number of
// loads (missing ones go, out of range, to a dump block), so one compile-time vmcnt wait per
// step orders everything; nine steps per chunk and three ring stages make the stage of a step a
// compile-time constant of the unrolled tap loop.
#include <cstdio>

#include <atomic>

#include "dma_common.hpp"

namespace relay {
namespace {

struct HaloGeom {
  int P, F;           // row pitch W + 1 and image pitch (H + 1) * P of the flat coordinate
  int Mflat;          // N * F flat output positions
  float rcp_p, rcp_f;
  int xblk;           // 16-row blocks per plane of a halo buffer
  int nxbuf;          // halo buffers: 2 when there are several channel chunks, else 1
  int ncc;            // channel chunks, C / CK
  int tab_slot;       // 16-byte slot of LDS where the pixel table starts (behind the ring and the epilogue staging)
  FastDiv fd_f, fd_xblk;            // division by F and by xblk
  FastDiv fd_tiles_m, fd_tiles_n;   // ... by the tile counts of the launched variant
};

constexpr int NSW = 3;         // filter ring stages (9 taps per chunk keep step % NSW compile-time)
constexpr int XS = 11 - NSW;   // taps of a chunk behind which the next chunk's halo is loaded

// HB: halo blocks a wave loads per issue slot (a halo holds at most XS * HB * waves blocks of 16 positions)
template <bool IS_I8, int WAVES_M, int WAVES_N, int TM, int TN, int KP, int HB = 1>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, 2) void conv3x3_halo_kernel(const ConvArgs a, const HaloGeom g) {
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int VE = IS_I8 ? 16 : 8;
  constexpr int ES = IS_I8 ? 1 : 2;
  constexpr int CK = KP * BKV * VE;
  constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
  constexpr int WTM = TM * 32, WTN = TN * 32;
  static_assert((BN / 16) % NW == 0, "filter staging blocks must divide over the waves");
  constexpr int WLP = BN / 16 / NW;      // filter blocks per plane per wave
  constexpr int LW = KP * WLP;           // filter loads per step per wave
  constexpr int L = LW + HB;             // loads per step per wave: filters + HB halo blocks
  constexpr int XN = XS * HB;            // halo blocks per wave
  constexpr int KSTEPS = KP * (BKV / 2);
  static_assert(L <= TM * TN * KSTEPS, "one load is issued behind each MFMA of a step");
  static_assert(XN + (NSW - 1) * L + 8 <= 63, "vmcnt is a 6-bit counter");
  constexpr int WPLANE = BN * BKV;       // 16-byte slots of one filter plane
  constexpr int WSTAGE = KP * WPLANE;
  constexpr int EP = WTN / 4 + 1;
  typedef typename Mma<IS_I8>::acc_t acc_t;

  extern __shared__ uint4 lds[];
  const int xplane = g.xblk * 64;                   // slots of one halo plane
  const int xbuf_slots = KP * xplane;
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) uint4*)(&lds[0]);
  const unsigned wring_base = lds_base + (unsigned)(g.nxbuf * xbuf_slots) * 16u;
  const unsigned dump_base = wring_base + (unsigned)(NSW * WSTAGE) * 16u;
  const uint4* wring = lds + g.nxbuf * xbuf_slots;

  // Every argument the kernel uses is asked for here, so that their scalar loads leave as one batch with one
  // wait; left to itself the compiler loads them where they are first used, and the prologue then waits
  // for five scalar-load round trips one after another.
  asm volatile("" ::"s"(a.x), "s"(a.w), "s"(a.y), "s"(a.res), "s"(a.bias), "s"(a.scale), "s"(a.shift), "s"(a.qbias));
  asm volatile("" ::"s"(a.N), "s"(a.H), "s"(a.W), "s"(a.C), "s"(a.K), "s"(a.Kp), "s"(a.flags), "s"(a.param_vec),
               "s"(a.n_major), "s"(a.xs_n));
  if constexpr (IS_I8)   // (the quantized tail's own arguments too)
    asm volatile("" ::"s"(a.lshift), "s"(a.rshift), "s"(a.round_add), "s"(a.qmode), "s"(a.clip_lo), "s"(a.clip_hi), "s"(a.qmult),
                 "s"(a.qshift));
  asm volatile("" ::"s"(g.P), "s"(g.F), "s"(g.Mflat), "s"(g.rcp_p), "s"(g.rcp_f), "s"(g.xblk), "s"(g.nxbuf), "s"(g.ncc),
               "s"(g.tab_slot), "s"(g.fd_f.mul), "s"(g.fd_f.shift), "s"(g.fd_xblk.mul), "s"(g.fd_xblk.shift),
               "s"(g.fd_tiles_m.mul), "s"(g.fd_tiles_m.shift), "s"(g.fd_tiles_n.mul), "s"(g.fd_tiles_n.shift));
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  const int tiles_m = (g.Mflat + BM - 1) / BM, tiles_n = (a.K + BN - 1) / BN;
  const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int tile_q = (int)fast_div((uint32_t)tile, a.n_major ? g.fd_tiles_m : g.fd_tiles_n);
  const int tile_n = a.n_major ? tile_q : tile - tile_q * tiles_n;
  const int tile_m = a.n_major ? tile - tile_q * tiles_m : tile_q;
  const int o0 = tile_m * BM, n0 = tile_n * BN;
  const int n_0 = (int)fast_div((uint32_t)o0, g.fd_f);  // (uniform) image and in-image position of the tile's first position
  const int rem_0 = o0 - n_0 * g.F;

  // ---- first loads out as early as possible: the epilogue constants (oldest, so that nothing ever waits for
  //      them longer than for a ring load), then the filters of step 0, which need no decoding.  Every issue
  //      slot, here and in the loop, holds L loads (a dump load stands in where there is none), and
  //      the order of the slots is what the waits count on: filters of step 0, the halo of chunk 0,
  //      filters of step 1.
  const int srow = lane >> 2, sphys = lane & 3;
  constexpr int CG = WTN / 8;  // lanes per pixel row in the epilogue
  const int ech = n0 + wn * WTN + (lane % CG) * 8;
  RawLaneParams rawp;
  fetch_lane_params<IS_I8>(a, ech, rawp);
  unsigned w_off[WLP];
#pragma unroll
  for (int j = 0; j < WLP; ++j) {
    const int row = (wave * WLP + j) * 16 + srow;
    const int kvl = sphys ^ lds_swizzle(row);
    const int ch = n0 + row;
    w_off[j] = ch < a.K ? (unsigned)((ch * a.Kp + kvl * VE) * ES) : kOob;
  }
  const intx4 rs_x = make_rsrc(a.x, (unsigned)((size_t)a.N * a.xs_n * ES));
  const intx4 rs_w = make_rsrc(a.w, (unsigned)((size_t)a.K * a.Kp * ES));
  auto issue_filters = [&](int s) {  // the filters of step (0, s), s < NSW - 1, and the slot's dump loads
#pragma unroll
    for (int i = 0; i < LW; ++i) {
      const int plane = i / WLP, j = i % WLP;
      lds_dma16(rs_w, wring_base + (unsigned)(s * WSTAGE + plane * WPLANE + (wave * WLP + j) * 64) * 16u,
                w_off[j] == kOob ? kOob : w_off[j] + (unsigned)((s * a.C + plane * (BKV * VE)) * ES));
    }
#pragma unroll
    for (int h = 0; h < HB; ++h) lds_dma16(rs_x, dump_base, kOob);
  };
  issue_filters(0);

  // ---- pixel table: for each of the halo's xblk * 16 flat positions the index (n * H + row) * W + col of
  //      the input pixel there, or ~0 where the position is padding.  One decode per thread (or two)
  //      instead of one per load and per stored pixel: the halo loads below look their rows up here, and so
  //      does the epilogue, because the output pixel of flat position o is the input pixel of o + P + 1.
  unsigned* ptab = reinterpret_cast<unsigned*>(lds + g.tab_slot);
  for (int r = tid; r < g.xblk * 16; r += NW * 64) {
    int dn, r1, rowi, coli;
    small_divmod(rem_0 + r, g.F, g.rcp_f, dn, r1);
    small_divmod(r1, g.P, g.rcp_p, rowi, coli);
    const int n = n_0 + dn;
    ptab[r] = (n < a.N && rowi >= 1 && coli >= 1) ? (unsigned)((n * a.H + rowi - 1) * a.W + coli - 1) : ~0u;
  }
  // (the table is LDS traffic only: the loads already in flight are not waited for here)
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();

  // ---- this lane's part of a halo: block (t * NW + wave) of the KP * xblk blocks, for t < XN; the load of
  //      chunk 0's block goes out as soon as its address is known
  unsigned x_off[XN];    // byte offset of the 16 bytes this lane fetches (chunk 0), or out of range
  unsigned x_dst[XN];    // LDS byte offset inside a halo buffer
  unsigned x_live = 0;   // bit t: the block exists (else the load goes to the dump block)
  unsigned x_px[XN];     // (all table reads first: one wait for all of them)
#pragma unroll
  for (int t = 0; t < XN; ++t) {
    const int b = t * NW + wave;
    const int plane = (int)fast_div((uint32_t)b, g.fd_xblk), blk = b - plane * g.xblk;
    x_px[t] = ptab[plane < KP ? blk * 16 + srow : 0];
  }
#pragma unroll
  for (int t = 0; t < XN; ++t) {
    const int b = t * NW + wave;
    const int plane = (int)fast_div((uint32_t)b, g.fd_xblk), blk = b - plane * g.xblk;
    const bool live = plane < KP;
    const int row = blk * 16 + srow;
    const int kvl = sphys ^ lds_swizzle(row);
    const unsigned px = x_px[t];
    x_off[t] = (live && px != ~0u) ? (unsigned)((px * a.C + plane * (BKV * VE) + kvl * VE) * ES) : kOob;
    x_dst[t] = (unsigned)((plane * g.xblk + blk) * 64) * 16u;
    if (live) x_live |= 1u << t;
    lds_dma16(rs_x, live ? lds_base + x_dst[t] : dump_base, live ? x_off[t] : kOob);
  }
#pragma unroll
  for (int s = 1; s < NSW - 1; ++s) issue_filters(s);

  // the i-th load of the issue slot behind step (cc, t): filters of step (cc, t) + NSW - 1, then
  // blocks t * HB ... of the halo of chunk cc + 1
  auto issue_one = [&](int cc, int t, int i) {
    if (i < LW) {
      const int tw = (t + NSW - 1) % 9, ccw = cc + (t + NSW - 1) / 9;  // tap and chunk of the step being fetched
      const int plane = i / WLP, j = i % WLP;
      const bool live = ccw < g.ncc;
      const unsigned voff = live ? w_off[j] + (unsigned)((tw * a.C + ccw * CK + plane * (BKV * VE)) * ES) : kOob;
      lds_dma16(rs_w, wring_base + (unsigned)(((t + NSW - 1) % NSW) * WSTAGE + plane * WPLANE + (wave * WLP + j) * 64) * 16u, voff);
    } else {
      const int xt = t < XS ? t * HB + (i - LW) : 0;   // which of this wave's halo blocks
      const bool live = t < XS && ((x_live >> xt) & 1u) && cc + 1 < g.ncc;
      const unsigned voff = (live && x_off[xt] != kOob) ? x_off[xt] + (unsigned)((cc + 1) * CK * ES) : kOob;
      const unsigned dst = live ? lds_base + (unsigned)((((cc + 1) & 1) * (g.nxbuf - 1)) * xbuf_slots) * 16u + x_dst[xt] : dump_base;
      lds_dma16(rs_x, dst, voff);
    }
  };

  acc_t acc[TN][TM];
#pragma unroll
  for (int tn = 0; tn < TN; ++tn)
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tn][tm][v] = 0;

  LaneParams lp;
  finish_lane_params<IS_I8>(rawp, lp);

  const int lrow = lane & 31, lhalf = lane >> 5;
  const int xrow0 = wm * WTM + lrow;  // halo row of this lane's first pixel at tap (0, 0)
  for (int cc = 0; cc < g.ncc; ++cc) {
    const uint4* xb = lds + ((cc & 1) * (g.nxbuf - 1)) * xbuf_slots;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
      // step (cc, t) has landed once only the loads of the NSW - 2 issue slots after its own are pending
      wait_loads<(NSW - 2) * L>();
      __builtin_amdgcn_s_barrier();
      const uint4* ws = wring + (t % NSW) * WSTAGE;
      const int xrow = xrow0 + (t / 3) * g.P + (t % 3);  // the tap is a shift of the halo rows
      const int xs = lds_swizzle(xrow);                  // unchanged by the + 32 of the next block
      uint4 wf[KSTEPS][TN], xf[KSTEPS][TM];
#pragma unroll
      for (int k = 0; k < KSTEPS; ++k) {
        const int kq = 2 * (k & 1) + lhalf;
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) wf[k][tn] = ws[(k >> 1) * WPLANE + lds_slot(wn * WTN + tn * 32 + lrow, kq)];
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) xf[k][tm] = xb[(k >> 1) * xplane + (xrow + tm * 32) * BKV + (kq ^ xs)];
      }
#pragma unroll
      for (int k = 0; k < KSTEPS; ++k)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
          for (int tm = 0; tm < TM; ++tm) {
            acc[tn][tm] = Mma<IS_I8>::mma(wf[k][tn], xf[k][tm], acc[tn][tm]);
            const int i = (k * TN + tn) * TM + tm;  // one load rides behind each MFMA
            if (i < L) {
              __builtin_amdgcn_sched_barrier(0);
              issue_one(cc, t, i);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
    }
  }

  // ---- epilogue: as in the implicit-GEMM kernel, with the flat position decoded back to a pixel
  wait_loads<0>();               // the trailing out-of-range loads still write zeros
  __builtin_amdgcn_s_barrier();  // every wave is done reading
  uint4* stg = lds + wave * (32 * EP);
  constexpr int PPI = 64 / CG;
  const int epix = lane / CG, ecg = lane % CG;
  const bool vec_ok = (a.K & 7) == 0;
  const OutLoc ol{nullptr, 0, 0};  // this kernel stores plain tensors only
  // the output pixels of this lane (the output pixel of a flat position o is the table's entry for o + P + 1),
  // read together, and all its residual vectors: in flight together, behind the transpositions below
  constexpr int ITS = 32 / PPI;
  const bool pre_res = (a.flags & F_RES) && vec_ok;
  unsigned mpix[TM][ITS];
  uint4 resv[TM][ITS];
#pragma unroll
  for (int tm = 0; tm < TM; ++tm)
#pragma unroll
    for (int it = 0; it < ITS; ++it) mpix[tm][it] = ptab[wm * WTM + tm * 32 + it * PPI + epix + g.P + 1];
  if (pre_res) {
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int it = 0; it < ITS; ++it)
        resv[tm][it] = (mpix[tm][it] != ~0u && ech < a.K) ? load_residual8<IS_I8>(a, (int)mpix[tm][it], ech)
                                                           : make_uint4(0u, 0u, 0u, 0u);
  }
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) {
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        uint4 v;
        v.x = as_u32(acc[tn][tm][4 * q4]);
        v.y = as_u32(acc[tn][tm][4 * q4 + 1]);
        v.z = as_u32(acc[tn][tm][4 * q4 + 2]);
        v.w = as_u32(acc[tn][tm][4 * q4 + 3]);
        stg[lrow * EP + tn * 8 + 2 * q4 + lhalf] = v;
      }
    // same wave wrote what it now reads: LDS operations of a wave execute in order
#pragma unroll
    for (int it = 0; it < 32 / PPI; ++it) {
      const int pix = it * PPI + epix;
      const uint4 lo = stg[pix * EP + ecg * 2], hi = stg[pix * EP + ecg * 2 + 1];
      const unsigned raw[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      const unsigned m = mpix[tm][it];
      if (m == ~0u || ech >= a.K) continue;  // not a pixel, or past Cout
      finish_store8<IS_I8, false>(a, raw, (int)m, ech, lp, ol, vec_ok, pre_res, resv[tm][it]);
    }
  }
}

struct HaloTile {
  int waves_m, waves_n, tm, tn, hb;
  constexpr int bm() const { return waves_m * tm * 32; }
  constexpr int bn() const { return waves_n * tn * 32; }
};
// 128 x 64, 64 x 64, 256 x 64 (four waves of 64 x 64, a third less LDS operand traffic per matrix instruction:
// a layer whose 128-position tiles would take the chip two rounds takes one) and 128 x 128
constexpr HaloTile kHalo[] = {{2, 2, 2, 1, 1}, {2, 2, 1, 1, 1}, {4, 1, 2, 2, 2}, {2, 2, 2, 2, 1}};
constexpr int kNumHalo = 4;

int chunk_planes(const ConvArgs& a, bool is_i8, int v) {
  const int ve = is_i8 ? 16 : 8;
  // the 64 x 64 tile takes 256-byte chunks (half the barriers per product) where the channel count allows and
  // the halo still fits the load slots
  if (v == 1 && a.C % (4 * BKV * ve) == 0 && 4 * ((kHalo[v].bm() + 2 * (a.W + 1) + 2 + 15) / 16) <= XS * kHalo[v].hb * 4)
    return 4;
  return a.C % (2 * BKV * ve) == 0 ? 2 : 1;
}

bool make_geom(const ConvArgs& a, bool is_i8, int v, HaloGeom& g, size_t& lds_bytes) {
  const int kp = chunk_planes(a, is_i8, v), ve = is_i8 ? 16 : 8;
  g.P = a.W + 1;
  g.F = (a.H + 1) * g.P;
  if ((long)a.N * g.F > 0x3fffffffL || g.F >= (1 << 21)) return false;
  g.Mflat = a.N * g.F;
  g.rcp_p = 1.0f / (float)g.P;
  g.rcp_f = 1.0f / (float)g.F;
  const int rows = kHalo[v].bm() + 2 * g.P + 2;
  g.xblk = (rows + 15) / 16;
  g.ncc = a.C / (kp * BKV * ve);
  g.nxbuf = g.ncc > 1 ? 2 : 1;
  g.fd_f = make_fastdiv((uint32_t)g.F);
  g.fd_xblk = make_fastdiv((uint32_t)g.xblk);
  if (kp * g.xblk > XS * kHalo[v].hb * 4) return false;  // a halo must fit the load slots of XS steps x 4 waves
  const int nw = kHalo[v].waves_m * kHalo[v].waves_n;
  const size_t ring = (size_t)g.nxbuf * kp * g.xblk * 64 + (size_t)NSW * kp * kHalo[v].bn() * BKV + 64;
  const size_t epi = (size_t)nw * 32 * (kHalo[v].tn * 32 / 4 + 1);
  g.tab_slot = (int)(ring > epi ? ring : epi);
  lds_bytes = ((size_t)g.tab_slot + (size_t)g.xblk * 4) * 16;  // + 4 bytes per halo position
  return lds_bytes <= 160 * 1024;
}

template <bool IS_I8, int WM, int WN, int TM, int TN, int KP, int HB = 1>
hipError_t launch_halo_one(const ConvArgs& a, const HaloGeom& g, size_t lds_bytes, hipStream_t st) {
  auto kern = conv3x3_halo_kernel<IS_I8, WM, WN, TM, TN, KP, HB>;
  static std::atomic<bool> raised{false};  // dynamic LDS above the default limit has to be asked for once per kernel
  if (!raised.load(std::memory_order_acquire)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                             160 * 1024);
    if (e != hipSuccess) return e;
    raised.store(true, std::memory_order_release);
  }
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  const int tiles_m = (g.Mflat + BM - 1) / BM, tiles_n = (a.K + BN - 1) / BN;
  HaloGeom gl = g;
  gl.fd_tiles_m = make_fastdiv((uint32_t)tiles_m);
  gl.fd_tiles_n = make_fastdiv((uint32_t)tiles_n);
  hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(64 * WM * WN), lds_bytes, st, a, gl);
  return hipGetLastError();
}

template <bool IS_I8>
hipError_t launch_halo_typed(const ConvArgs& a, const HaloGeom& g, size_t lds_bytes, int v, int kp, hipStream_t st) {
  if (v == 0) return kp == 2 ? launch_halo_one<IS_I8, 2, 2, 2, 1, 2>(a, g, lds_bytes, st)
                             : launch_halo_one<IS_I8, 2, 2, 2, 1, 1>(a, g, lds_bytes, st);
  if (v == 2) return kp == 2 ? launch_halo_one<IS_I8, 4, 1, 2, 2, 2, 2>(a, g, lds_bytes, st)
                             : launch_halo_one<IS_I8, 4, 1, 2, 2, 1, 2>(a, g, lds_bytes, st);
  if (v == 3) return kp == 2 ? launch_halo_one<IS_I8, 2, 2, 2, 2, 2>(a, g, lds_bytes, st)
                             : launch_halo_one<IS_I8, 2, 2, 2, 2, 1>(a, g, lds_bytes, st);
  if (kp == 4) return launch_halo_one<IS_I8, 2, 2, 1, 1, 4>(a, g, lds_bytes, st);
  return kp == 2 ? launch_halo_one<IS_I8, 2, 2, 1, 1, 2>(a, g, lds_bytes, st)
                 : launch_halo_one<IS_I8, 2, 2, 1, 1, 1>(a, g, lds_bytes, st);
}

}  // namespace

int conv_halo_variant_count() { return kNumHalo; }

// 3x3, stride 1, pad 1, plain NHWC, whole chunks of channels, deterministic rounding.
bool conv_halo_supported(const ConvArgs& a, bool is_i8, int v) {
  if (v < 0 || v >= kNumHalo) return false;
  const int es = is_i8 ? 1 : 2, ve = is_i8 ? 16 : 8;
  if (a.R != 3 || a.S != 3 || a.sh != 1 || a.sw != 1 || a.ph != 1 || a.pw != 1) return false;
  if (a.xs_w != a.C || a.xs_h != a.W * a.C || a.xs_n != a.H * a.W * a.C) return false;
  if (a.C % (BKV * ve) != 0 || a.round_mode == ROUND_STOCHASTIC || a.nseg) return false;
  if ((size_t)a.N * a.xs_n * es > 0x7fffffffu || (size_t)a.K * a.Kp * es > 0x7fffffffu) return false;
  HaloGeom g;
  size_t lds_bytes;
  return make_geom(a, is_i8, v, g, lds_bytes);
}

// The variant the heuristic takes, or -1 to leave the layer to the implicit-GEMM kernel.  Measured on
// the ResNet shapes at batch 32 (fp16 / int8): 128 channels at 28 x 28 12.9 against 15.1 us / 9.2
// against 9.6, 256 channels at 14 x 14 12.4 against 16.4 / 8.6 against 10.2; even at 64 fp16 channels
// (int8, batch 16: 7.1 against 7.9; fp16, batch 32, 813 tiles: 17.4 against 18.3, the whole ResNet-18
// stack 0.8 % faster), slower at 7 x 7 (a quarter of the flat positions are not pixels) and outside
// the range of tile counts where both kernels get two workgroups per CU.
int conv_halo_pick(const ConvArgs& a, bool is_i8) {
  const bool thin = !is_i8 && a.C == 64 && a.K <= 64;   // (wide images too: 112 x 112 at batch 32 57.4 against 62.8 us, 224 x 224 216.8 against 226.5)
  // fp16, 512 and more channels at 7 x 7 and below: the 64 x 64 tile with 256-byte chunks (a third of the global->LDS
  // traffic of the implicit GEMM's 64 x 64 tile; 512 -> 512 at batch 32: 14.9 against 16.4 us)
  if (!is_i8 && a.C >= 512 && a.W <= 7 && chunk_planes(a, is_i8, 1) == 4 && conv_halo_supported(a, is_i8, 1)) {
    const long t64 = (((long)a.N * (a.H + 1) * (a.W + 1) + 63) / 64) * ((a.K + 63) / 64);
    if (t64 >= 190 && t64 <= 512) return 1;
  }
  if (a.C < 64 || (a.W > 56 && !thin) || !conv_halo_supported(a, is_i8, 0)) return -1;
  const long flat = (long)a.N * (a.H + 1) * (a.W + 1);
  const long t128 = ((flat + 127) / 128) * ((a.K + 63) / 64);
  // (fp16, 256 channels and more: also on layers of thousands of tiles -- VGG-16 at batch 32: 256 -> 512 at 28 x 28
  // 68.8 against 76.9 us, 512 -> 512 129.3 against 142.7, 256 -> 256 at 56 x 56 147.4 against 151.3; 64 -> 64 at any
  // size: 31.3 against 33.6 us at 56 x 56, batch 64)
  const bool any_size = !is_i8 && (a.C >= 256 || thin);
  const long cap = is_i8 ? 512 : (any_size ? (1L << 40) : (a.C == 64 ? 1024 : 512));
  if (t128 < 190 || t128 > cap) return -1;
  // very many tiles of wide layers: 128 x 128 tiles, two thirds of the LDS operand traffic per matrix
  // instruction (256 -> 256 at 56 x 56, batch 32: 130.0 against 147.1 us; a loss at 844 tiles, 512 at 28 x 28)
  const long t128sq = ((flat + 127) / 128) * ((a.K + 127) / 128);
  if (!is_i8 && a.C >= 256 && t128sq >= 1500 && conv_halo_supported(a, is_i8, 3)) return 3;
  // 64 -> 64 channels in fp16 where the 128-position tiles would take the chip between one and about three
  // rounds of its 512 workgroup slots: the 256-position tile halves the rounds (56 x 56 at batch 32: 15.0
  // against 16.2 us)
  if (thin && t128 > 512 && t128 <= 1700 && conv_halo_supported(a, is_i8, 2)) return 2;
  return 0;
}

void conv_halo_kernel_name(const ConvArgs& a, bool is_i8, int v, char* buf, size_t len) {
  snprintf(buf, len, "conv3x3_halo_kernel<%s, %d, %d, %d, %d, %d, %d>", is_i8 ? "true" : "false", kHalo[v].waves_m,
           kHalo[v].waves_n, kHalo[v].tm, kHalo[v].tn, chunk_planes(a, is_i8, v), kHalo[v].hb);
}

hipError_t launch_conv_halo(const ConvArgs& a, bool is_i8, int v, hipStream_t st) {
  HaloGeom g;
  size_t lds_bytes;
  if (!make_geom(a, is_i8, v, g, lds_bytes)) return hipErrorInvalidValue;
  const int kp = chunk_planes(a, is_i8, v);
  return is_i8 ? launch_halo_typed<true>(a, g, lds_bytes, v, kp, st) : launch_halo_typed<false>(a, g, lds_bytes, v, kp, st);
}

}  // namespace relay
