// Implicit-GEMM conv2d for gfx950: MFMA main loop fed by direct global->LDS loads through a
// multi-stage LDS ring, fused epilogue (paper Section 4.1 / 4.2).
//
// GEMM view: rows m = (image, p, q) output pixels, columns = output channels, reduction
// kk = (r, s, c).  NHWC activations and [k][r][s][c] filters are both contiguous along the
// reduction axis and move as 16-byte k-vectors.  A workgroup owns BM pixels x BN channels;
// a wave owns TM x TN MFMA blocks of 32x32 (filters are the A operand).
//
// Staging: per 64-byte reduction chunk every wave issues `buffer_load_dwordx4 ... lds`
// instructions, each moving 16 tile rows x 64 B straight into LDS (lane i writes 16 bytes
// at base + 16*i), no VGPRs involved.  The LDS bank swizzle is applied on the global side:
// lane i fetches the k-vector that belongs in its fixed LDS slot.  Filter taps that fall in
// the padding, rows past the end of the tensor and channels past Cout get a buffer offset
// beyond num_records; the buffer unit then writes zeros (checked on hardware), so the MFMA
// loop has no special cases.  NS ring stages keep NS-1 chunks in flight behind one barrier
// per chunk.  The loads are inline asm on purpose: the compiler, not seeing LDS written,
// does not drain the memory pipeline before every LDS read; ordering is by the explicit
// vmcnt waits and barriers below.  The texture addresser takes 64 B/clk per CU, about as
// long per chunk as the MFMAs of a 256x128 tile take, so the loads of chunk kc+NS-1 are
// issued one at a time between the MFMAs of chunk kc instead of in a burst after the
// barrier, where all waves would queue for the addresser while the matrix pipe idles.
//
// Epilogue: accumulators go through LDS once (wave-private, 32 pixels at a time) so that a
// lane ends up with 8 consecutive channels of one pixel: per-channel constants are then the
// same for every pixel a lane handles, the residual is one 16-byte load and the result one
// 16-byte (fp16) or 8-byte (int8) store in full NHWC rows.
//
// Needs C to be a whole number of chunks (32 halves / 64 int8) and R*S <= 32; other shapes
// go to the register-staged kernel in conv_igemm.hip.
#include <cstdio>
#include <type_traits>

#include "dma_common.hpp"

namespace relay {
namespace {

// KP = 64-byte planes per ring chunk (a chunk covers KP*64 bytes of reduction; each plane is
// a [rows][64 B] sub-tile with its own swizzle, because 128-byte LDS rows cannot be read
// conflict-free).  More planes = fewer barriers and fewer exposed LDS latencies per MFMA.
// SK = waves that share one accumulator tile and split the k-steps of every chunk between
// them (their partial sums meet in LDS before the epilogue).  A wave then owns a SK times
// larger tile for the same workgroup tile, which cuts the LDS operand reads per MFMA -- the
// resource the small tiles are bound by.
// STOCH: the stochastic rounding of the quantized epilogue (its generator costs registers, so it is an
// instantiation of its own; the deterministic rules are one host-computed addend).
// Arrival counters of different tiles sit 256 bytes apart: device-scope atomics on one line
// are served one after another.
constexpr int kCntStride = 64;

template <bool IS_I8>
using acc_t_scalar = typename std::conditional<IS_I8, int, float>::type;

// EXT: the instantiation that can split a tile's reduction over workgroups and store output
// channel segments.  Both are rare; kept out of the plain kernel because even as untaken uniform
// branches they cost it about 1 % each (registers held across the main loop, code size).
// POOL: the tile is the 15 x 17 patch of conv outputs under a 7 x 8 block of 3x3/s2/p1 max-pool
// outputs (255 of 256 rows); the finished patch goes to LDS and only the pooled block is stored.
template <bool IS_I8, int WAVES_M, int WAVES_N, int TM, int TN, int NS, int KP, int SK, bool STOCH, bool EXT,
          bool POOL = false>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N * SK,
                             // two workgroups per CU where their LDS rings fit side by side
                             (NS * KP * (WAVES_M * TM + WAVES_N * TN) * 32 * 64 <= 80 * 1024 ? 2 : 1))
    void igemm_dma_kernel(const ConvArgs a) {
  constexpr int NW = WAVES_M * WAVES_N * SK;
  static_assert(SK == 1 || (SK == 2 && KP == 2 && TM % 2 == 0), "k-split pairs take one 64-byte plane each");
  constexpr int VE = IS_I8 ? 16 : 8;
  constexpr int ES = IS_I8 ? 1 : 2;
  constexpr int CK = KP * BKV * VE;
  constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
  constexpr int WTM = TM * 32, WTN = TN * 32;
  constexpr int XB = BM / 16, WB = BN / 16;  // 1 KiB staging blocks: 16 rows x 64 B
  static_assert(XB % NW == 0 && WB % NW == 0, "staging blocks must divide over the waves");
  constexpr int XL = XB / NW, WL = WB / NW;    // loads per plane per wave
  constexpr int LPC = KP * (XL + WL);          // loads per chunk per wave
  constexpr int PLANE = (BM + BN) * BKV;       // 16-byte slots per plane
  constexpr int STAGE = KP * PLANE;            // ... per ring stage
  constexpr int KSTEPS = KP * (BKV / 2);       // MFMA k-steps per chunk
  static_assert((NS - 1) * LPC <= 63, "vmcnt is a 6-bit counter");
  constexpr int KSW = KSTEPS / SK;             // ... of which this wave runs KSW
  // one load is issued behind each MFMA of a chunk; a two-wave tile has more loads than MFMAs and issues the rest behind the last one
  static_assert(LPC <= TM * TN * KSW || (SK == 1 && !(TM + TN <= 4 && KP >= 4)), "the carried-MFMA schedule issues loads behind MFMAs only");
  constexpr int EP = WTN / 4 + 1;  // epilogue staging pitch (16-byte slots) of one pixel row, padded
  constexpr int XCH = SK == 2 ? (TM / 2) * TN * 4 * 64 : 0;  // slots a wave hands to its k-split partner
  static_assert(NW * (32 * EP + XCH) <= NS * STAGE, "epilogue staging reuses the ring");
  typedef typename Mma<IS_I8>::acc_t acc_t;

  constexpr int PDY = 15, PDX = 17;                 // conv patch of a pooled 7 x 8 block
  // the finished patch in LDS, [conv pixel][channel] in the output type; 8 bytes of padding per row
  // spread the accumulator layout's writes (32 lanes, 32 consecutive rows, one 4-channel group) over the banks
  constexpr int PPITCH = POOL ? BN * ES + 8 : 0;
  static_assert(!POOL || (BM >= PDY * PDX && SK == 1 && !EXT && !STOCH && WAVES_N == 1), "pooled tiles hold one 15 x 17 patch");
  static_assert(BM * PPITCH <= NS * STAGE * 16, "the patch reuses the ring");
  __shared__ uint4 ring[NS * STAGE];
  __shared__ float pool_cst[POOL ? 2 * BN : 1];  // pooled tiles: the epilogue constants of the tile's channels

  // The arguments of the prologue are asked for here, so that their scalar loads leave as one batch with
  // one wait; left to itself the compiler loads them where they are first used and the prologue waits
  // for several scalar-load round trips one after another.
  asm volatile("" ::"s"(a.x), "s"(a.w), "s"(a.bias), "s"(a.scale), "s"(a.shift), "s"(a.qbias));
  asm volatile("" ::"s"(a.N), "s"(a.H), "s"(a.W), "s"(a.C), "s"(a.K), "s"(a.R), "s"(a.S), "s"(a.sh), "s"(a.sw), "s"(a.ph),
               "s"(a.pw), "s"(a.Ho), "s"(a.Wo), "s"(a.xs_n), "s"(a.xs_h), "s"(a.xs_w), "s"(a.rcp_wo), "s"(a.rcp_ho),
               "s"(a.tap_spread), "s"(a.param_vec), "s"(a.n_major), "s"(a.M), "s"(a.Kred), "s"(a.Kp), "s"(a.flags));
  asm volatile("" ::"s"(a.fd_wo.mul), "s"(a.fd_wo.shift), "s"(a.fd_howo.mul), "s"(a.fd_howo.shift), "s"(a.fd_tiles_m.mul),
               "s"(a.fd_tiles_m.shift), "s"(a.fd_tiles_n.mul), "s"(a.fd_tiles_n.shift));
  if constexpr (IS_I8)   // (the quantized tail's own arguments too: asked for at its first use they cost it a scalar-load round trip per branch)
    asm volatile("" ::"s"(a.res), "s"(a.y), "s"(a.lshift), "s"(a.rshift), "s"(a.round_add), "s"(a.qmode), "s"(a.clip_lo), "s"(a.clip_hi),
                 "s"(a.qmult), "s"(a.qshift));
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wk = wave / (WAVES_M * WAVES_N), wsub = wave % (WAVES_M * WAVES_N);
  const int wm = wsub % WAVES_M, wn = wsub / WAVES_M;
  const int tiles_m = POOL ? a.N * a.pool_tiles_img : (a.M + BM - 1) / BM, tiles_n = (a.K + BN - 1) / BN;
  // with a split reduction consecutive workgroups (same XCD) share a tile
  const int nsplit = (EXT && a.split > 1) ? a.split : 1;
  const int wg = xcd_remap(blockIdx.x, tiles_m * tiles_n * nsplit);
  const int tile = wg / nsplit, ks = wg - tile * nsplit;
  const int tile_q = (int)fast_div((uint32_t)tile, a.n_major ? a.fd_tiles_m : a.fd_tiles_n);
  const int tile_n = a.n_major ? tile_q : tile - tile_q * tiles_n;
  const int tile_m = a.n_major ? tile - tile_q * tiles_m : tile_q;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // ---- staging role of this lane inside a 16-row block: row srow, physical slot sphys.
  //      The tile's first pixel is decoded once (uniform); rows are small offsets from it.
  const int srow = lane >> 2, sphys = lane & 3;
  const int HoWo = a.Ho * a.Wo;
  const int n_0 = (int)fast_div((uint32_t)m0, a.fd_howo);
  const int rem_0 = m0 - n_0 * HoWo;
  const int p_0 = (int)fast_div((uint32_t)rem_0, a.fd_wo);
  const int q_0 = rem_0 - p_0 * a.Wo;
  // (pooled tiles: image, and row / column of the 7 x 8 block of pooled outputs inside it)
  int pool_n = 0, pool_i = 0, pool_j = 0;
  if constexpr (POOL) {
    pool_n = (int)fast_div((uint32_t)tile_m, a.fd_pool_img);
    const int rem = tile_m - pool_n * a.pool_tiles_img;
    pool_i = (int)fast_div((uint32_t)rem, a.fd_pool_row);
    pool_j = rem - pool_i * a.pool_tiles_row;
  }
  int x_off[XL];        // byte offset of tap (0,0), channel 0 of the row's k-vector
  unsigned x_taps[XL];  // bit t set: tap t of this row lies inside the image
#pragma unroll
  for (int j = 0; j < XL; ++j) {
    const int row = (wave * XL + j) * 16 + srow;
    const int kvl = sphys ^ lds_swizzle(row);
    int dp, q, dn, p, n;
    bool row_ok;
    if constexpr (POOL) {  // row = dy * 17 + dx of the patch whose corner is conv output (14 i - 1, 16 j - 1)
      const int dy = row / PDX, dx = row - dy * PDX;
      p = 2 * 7 * pool_i - 1 + dy;
      q = 2 * 8 * pool_j - 1 + dx;
      n = pool_n;
      row_ok = dy < PDY && (unsigned)p < (unsigned)a.Ho && (unsigned)q < (unsigned)a.Wo;
      (void)dp;
      (void)dn;
    } else {
      small_divmod(q_0 + row, a.Wo, a.rcp_wo, dp, q);
      small_divmod(p_0 + dp, a.Ho, a.rcp_ho, dn, p);
      n = n_0 + dn;
      row_ok = m0 + row < a.M;
    }
    const int ih0 = p * a.sh - a.ph, iw0 = q * a.sw - a.pw;
    // filter rows [rlo, rhi) and columns [clo, chi) fall inside the image: the tap mask is the
    // column run replicated at every valid row (a product, the runs do not overlap)
    const int rlo = max(0, -ih0), rhi = min(a.R, a.H - ih0);
    const int clo = max(0, -iw0), chi = min(a.S, a.W - iw0);
    const unsigned colbits = (unsigned)((1ull << max(chi, 0)) - 1ull) & ~(unsigned)((1ull << clo) - 1ull);
    const unsigned rows = a.tap_spread & (unsigned)((1ull << (max(rhi, 0) * a.S)) - 1ull) &
                          ~(unsigned)((1ull << (rlo * a.S)) - 1ull);
    const unsigned taps = (rhi > rlo && chi > clo) ? colbits * rows : 0u;
    x_taps[j] = row_ok ? taps : 0u;
    x_off[j] = (n * a.xs_n + ih0 * a.xs_h + iw0 * a.xs_w + kvl * VE) * ES;
  }
  unsigned w_off[WL];
#pragma unroll
  for (int j = 0; j < WL; ++j) {
    const int row = (wave * WL + j) * 16 + srow;
    const int kvl = sphys ^ lds_swizzle(row);
    const int ch = n0 + row;
    w_off[j] = ch < a.K ? (unsigned)((ch * a.Kp + kvl * VE) * ES) : kOob;
  }
  const intx4 rs_x = make_rsrc(a.x, (unsigned)((size_t)a.N * a.xs_n * ES));
  const intx4 rs_w = make_rsrc(a.w, (unsigned)((size_t)a.K * a.Kp * ES));
  const unsigned ring_base = (unsigned)(size_t)(__attribute__((address_space(3))) uint4*)(&ring[0]);

  // this workgroup reduces chunks [kbeg, nchunks) of the layer's Kred / CK
  const int all_chunks = a.Kred / CK;
  const int per_split = (all_chunks + nsplit - 1) / nsplit;
  int kbeg = ks * per_split;
  int nchunks = min(all_chunks, kbeg + per_split);
  if constexpr (EXT) {
    if (a.seg_centre) {  // (uniform) a tile of a centre-tap segment reduces over that tap only (never split)
      int begin = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (i < a.nseg) {
          if (n0 >= begin && n0 < a.seg_end[i] && ((a.seg_centre >> i) & 1u)) {
            const int per_tap = a.C / CK;
            kbeg = ((a.R >> 1) * a.S + (a.S >> 1)) * per_tap;
            nchunks = kbeg + per_tap;
          }
          begin = a.seg_end[i];
        }
    }
  }
  // reduction position of the chunk being issued (wave-uniform)
  int is_tap = 0, is_r = 0, is_s = 0, is_c = 0, is_kc = kbeg;
  if (kbeg) {  // (uniform) position of the first chunk
    const int per_tap = a.C / CK;
    is_tap = kbeg / per_tap;
    is_c = (kbeg - is_tap * per_tap) * CK;
    is_r = is_tap / a.S;
    is_s = is_tap - is_r * a.S;
  }
  unsigned is_delta = (unsigned)((is_r * a.xs_h + is_s * a.xs_w + is_c) * ES), is_sbase = ring_base;
  bool is_live = is_kc < nchunks;
  // Small wave tiles (the short reductions) never issue a load for a chunk past the end of the
  // reduction: their loop ends in NS-1 iterations that only let the loads in flight run out.  The
  // large ones keep one loop shape for every chunk and issue all-out-of-range loads there instead
  // (a second copy of their loop body does not fit their register budget).
  constexpr bool RUNOUT = TM * TN < 8;
  // idx-th load of the chunk being issued: per plane XL activation blocks, then WL filter blocks
  auto issue_one = [&](int idx) {
    const int plane = idx / (XL + WL), i = idx % (XL + WL);
    const unsigned pbase = is_sbase + (unsigned)(plane * PLANE) * 16u;
    if (i < XL) {
      const unsigned voff = ((RUNOUT || is_live) && ((x_taps[i] >> is_tap) & 1u))
                                ? (unsigned)x_off[i] + is_delta + (unsigned)(plane * 64)
                                : kOob;
      lds_dma16(rs_x, pbase + (unsigned)((wave * XL + i) * 64) * 16u, voff);
    } else {
      const int j = i - XL;
      // (kOob + the chunk position stays out of range)
      const unsigned voff = (RUNOUT || is_live) ? w_off[j] + (unsigned)(is_kc * CK * ES + plane * 64) : kOob;
      lds_dma16(rs_w, pbase + (unsigned)(BM * BKV + (wave * WL + j) * 64) * 16u, voff);
    }
  };
  auto next_chunk = [&](int stage) {  // advance the issue position to the next chunk, landing in `stage`
    ++is_kc;
    is_c += CK;
    if (is_c == a.C) {
      is_c = 0;
      ++is_tap;
      if (++is_s == a.S) {
        is_s = 0;
        ++is_r;
      }
    }
    is_live = is_kc < nchunks;
    is_delta = (unsigned)((is_r * a.xs_h + is_s * a.xs_w + is_c) * ES);
    is_sbase = ring_base + (unsigned)(stage * STAGE) * 16u;
  };

  acc_t acc[TN][TM];
#pragma unroll
  for (int tn = 0; tn < TN; ++tn)
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tn][tm][v] = 0;

  // ---- epilogue constants of this lane: after the transposition it owns channels
  //      [ech, ech + 8) of whichever pixels it handles.  Their loads go out first; the values are
  //      used only after the ring loads below have been issued, which takes longer than the
  //      constants take to arrive.  (vmcnt counts these loads too; being older than every ring
  //      load they never make a wait for ring loads wait longer.)
  constexpr int CG = WTN / 8;  // lanes per pixel row in the epilogue
  const int ech = n0 + wn * WTN + (lane % CG) * 8;
  RawLaneParams rawp;
  fetch_lane_params<IS_I8>(a, ech, rawp);

#pragma unroll
  for (int s = 0; s < NS - 1; ++s) {
    if (!RUNOUT || is_live) {  // (uniform) a reduction shorter than the ring issues nothing for the chunks it does not have
#pragma unroll
      for (int i = 0; i < LPC; ++i) issue_one(i);
    }
    next_chunk(s + 1 == NS ? 0 : s + 1);
  }

  LaneParams lp;
  finish_lane_params<IS_I8>(rawp, lp);
  if constexpr (POOL) {  // lanes 0 .. BN/8-1 of a wave hold the constants of all BN channels between them
    if (wave == 0 && lane < BN / 8) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if constexpr (IS_I8) {
          pool_cst[lane * 8 + e] = __builtin_bit_cast(float, lp.ibias[e]);
        } else {
          pool_cst[lane * 8 + e] = lp.mul[e];
          pool_cst[BN + lane * 8 + e] = lp.add[e];
        }
      }
    }
  }

  const int lrow = lane & 31, lhalf = lane >> 5;
  int stage = 0;      // ring stage of chunk kc
  int fill = NS - 1;  // ring stage the chunk issued during this iteration lands in (set by next_chunk above)
  // Small wave tiles have too few MFMAs per k-step to cover the LDS latency of the next k-step's
  // operands, and right behind the barrier there is nothing to cover the first fetch at all.  So
  // they carry the second half of every chunk's MFMAs (operands already in registers) across the
  // barrier: those run while the first operands of the new chunk come in.  Order of the sums per
  // accumulator is unchanged.
  constexpr bool DEFER = TM + TN <= 4 && KP >= 4 && SK == 1;  // (measured: a gain with 8 k-steps per chunk, none with 4)
  constexpr int HK = DEFER ? KSW / 2 : 0;              // k-steps run in their own iteration
  constexpr int DK = DEFER ? KSW - HK : 1;             // k-steps carried into the next one
  uint4 wfd[DK][TN], xfd[DK][TM];
  bool carried = false;
  // One chunk of the reduction.  ISSUE: the loads of chunk kc+NS-1 ride behind this chunk's MFMAs
  // (every chunk but the last NS-1 of the reduction, which have nothing left to fetch); PENDING:
  // how many younger loads may still be in flight once this chunk's own have landed.
  auto chunk = [&](auto issue_tag, auto pending_tag) {
    constexpr bool ISSUE = decltype(issue_tag)::value;
    constexpr int PENDING = decltype(pending_tag)::value;
    wait_loads<PENDING>();
    __builtin_amdgcn_s_barrier();  // everyone's part of this chunk is in LDS; stage `fill` is free again
    const uint4* st = ring + stage * STAGE;
    // operand fetch of k-step k: plane k/2, k-vectors 2*(k%2) + lane/32
    auto fetch = [&](int k, uint4(&wf)[TN], uint4(&xf)[TM]) {
      const uint4* xs = st + (k >> 1) * PLANE;
      const uint4* ws = xs + BM * BKV;
      const int kq = 2 * (k & 1) + lhalf;
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) wf[tn] = ws[lds_slot(wn * WTN + tn * 32 + lrow, kq)];
#pragma unroll
      for (int tm = 0; tm < TM; ++tm) xf[tm] = xs[lds_slot(wm * WTM + tm * 32 + lrow, kq)];
    };
    // the MFMAs of one k-step; `slot` is the k-step's place in this iteration's MFMA sequence: one
    // ring load rides behind each of the first LPC MFMAs of an iteration
    auto mma_step = [&](int slot, const uint4(&wf)[TN], const uint4(&xf)[TM]) {
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
          acc[tn][tm] = Mma<IS_I8>::mma(wf[tn], xf[tm], acc[tn][tm]);
          const int i = (slot * TN + tn) * TM + tm;
          if (ISSUE && i < LPC) {
            __builtin_amdgcn_sched_barrier(0);  // keep the load behind this MFMA, not hoisted above all of them
            issue_one(i);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
    };
    const int k0 = wk * KSW;  // first k-step of this wave
    if constexpr (DEFER) {
      uint4 wf[HK][TN], xf[HK][TM];
#pragma unroll
      for (int k = 0; k < HK; ++k) fetch(k, wf[k], xf[k]);
      if (carried) {
#pragma unroll
        for (int k = 0; k < DK; ++k) mma_step(k, wfd[k], xfd[k]);
      } else if (ISSUE) {  // (first chunk) nothing carried: the loads of those slots go out in one go
#pragma unroll
        for (int i = 0; i < DK * TN * TM && i < LPC; ++i) issue_one(i);
      }
#pragma unroll
      for (int k = 0; k < DK; ++k) fetch(HK + k, wfd[k], xfd[k]);
#pragma unroll
      for (int k = 0; k < HK; ++k) mma_step(DK + k, wf[k], xf[k]);
      carried = true;
    } else {
      // operands of k-step k+PD are fetched before the MFMAs of k-step k run (PD+1 register sets);
      // the other small wave tiles fetch the whole chunk right behind the barrier
      constexpr int PD = (TM + TN <= 4 && KSW > 1) ? (KSW - 1 < 7 ? KSW - 1 : 7) : 1;
      uint4 wf[PD + 1][TN], xf[PD + 1][TM];
#pragma unroll
      for (int k = 0; k < PD && k < KSW; ++k) fetch(k0 + k, wf[k], xf[k]);
#pragma unroll
      for (int k = 0; k < KSW; ++k) {
        if (k + PD < KSW) fetch(k0 + k + PD, wf[(k + PD) % (PD + 1)], xf[(k + PD) % (PD + 1)]);
        mma_step(k, wf[k % (PD + 1)], xf[k % (PD + 1)]);
      }
      if constexpr (LPC > TM * TN * KSW) {
        if (ISSUE) {
#pragma unroll
          for (int i = TM * TN * KSW; i < LPC; ++i) issue_one(i);
        }
      }
    }
    if (ISSUE) {
      fill = fill + 1 == NS ? 0 : fill + 1;
      next_chunk(fill);
    }
    stage = stage + 1 == NS ? 0 : stage + 1;
  };
  using std::integral_constant;
  const int klen = max(nchunks - kbeg, 0);
  if constexpr (RUNOUT) {
    // all but the last NS-1 chunks: one more chunk is issued per chunk consumed, NS-2 stay in flight
    for (int kc = NS - 1; kc < klen; ++kc) chunk(std::true_type{}, integral_constant<int, (NS - 2) * LPC>{});
    // the last NS-1 (or fewer) chunks: nothing is issued any more, the loads in flight run out
    for (int left = min(klen, NS - 1) - 1; left >= 0; --left) {  // `left` chunks follow this one
      if (NS > 3 && left == 2) chunk(std::false_type{}, integral_constant<int, (NS > 3 ? 2 : 0) * LPC>{});
      else if (NS > 2 && left == 1) chunk(std::false_type{}, integral_constant<int, (NS > 2 ? 1 : 0) * LPC>{});
      else chunk(std::false_type{}, integral_constant<int, 0>{});
    }
  } else {
    for (int kc = 0; kc < klen; ++kc) chunk(std::true_type{}, integral_constant<int, (NS - 2) * LPC>{});
  }
  if constexpr (DEFER) {
    if (carried) {  // the last chunk's second half
#pragma unroll
      for (int k = 0; k < DK; ++k)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
          for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = Mma<IS_I8>::mma(wfd[k][tn], xfd[k][tm], acc[tn][tm]);
    }
  }

  // ---- epilogue.  Element v of a 32x32 accumulator block is channel 8*(v/4) + 4*(lane/32) + v%4
  //      of pixel lane%32.  Each wave transposes its blocks through a private LDS region.
  wait_loads<0>();               // (trailing out-of-range loads of the large tiles still write zeros into the ring)
  __builtin_amdgcn_s_barrier();  // every wave is done reading the ring
  constexpr int TM_E = SK == 2 ? TM / 2 : TM;  // accumulator block rows this wave finishes
  const int tm_lo = SK == 2 ? wk * TM_E : 0;
  if constexpr (SK == 2) {
    // the pair splits the tile: each wave hands the partner the half it does not finish
    uint4* give = ring + wave * XCH;
    const uint4* take = ring + (wave ^ (WAVES_M * WAVES_N)) * XCH;
#pragma unroll
    for (int t = 0; t < TM_E; ++t)
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int tm = (1 - wk) * TM_E + t;  // a block of the partner's half
          uint4 v;
          v.x = as_u32(wk ? acc[tn][t][4 * g] : acc[tn][TM_E + t][4 * g]);
          v.y = as_u32(wk ? acc[tn][t][4 * g + 1] : acc[tn][TM_E + t][4 * g + 1]);
          v.z = as_u32(wk ? acc[tn][t][4 * g + 2] : acc[tn][TM_E + t][4 * g + 2]);
          v.w = as_u32(wk ? acc[tn][t][4 * g + 3] : acc[tn][TM_E + t][4 * g + 3]);
          (void)tm;
          give[((t * TN + tn) * 4 + g) * 64 + lane] = v;
        }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the LDS writes are done
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int t = 0; t < TM_E; ++t)
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const uint4 v = take[((t * TN + tn) * 4 + g) * 64 + lane];
          const unsigned r[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if constexpr (IS_I8) {
              if (wk) acc[tn][TM_E + t][4 * g + e] += (int)r[e];
              else acc[tn][t][4 * g + e] += (int)r[e];
            } else {
              if (wk) acc[tn][TM_E + t][4 * g + e] += __builtin_bit_cast(float, r[e]);
              else acc[tn][t][4 * g + e] += __builtin_bit_cast(float, r[e]);
            }
          }
        }
  }
  if constexpr (POOL) {
    // Pooled tiles finish their accumulators where they are (element v of a block: pixel lane % 32,
    // channels 8 (v / 4) + 4 (lane / 32) + v % 4) and write the narrowed values, four channels at a
    // time, into the patch.
    char* patch_w = reinterpret_cast<char*>(ring);
    const ClipBounds qb = clip_bounds(a, a.flags & F_RELU);
    // (the quantized tail in both of its forms, chosen once for the tile)
    auto narrow = [&](auto sat) {
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int cb = tn * 32 + 8 * g + 4 * lhalf;  // first of the lane's four channels, within the tile
        const float4 c0 = *reinterpret_cast<const float4*>(pool_cst + cb);
        const float4 c1 = *reinterpret_cast<const float4*>(pool_cst + BN + cb);  // (fp16 only)
        const float m4[4] = {c0.x, c0.y, c0.z, c0.w}, a4[4] = {c1.x, c1.y, c1.z, c1.w};
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
          char* dst = patch_w + (wm * WTM + tm * 32 + lrow) * PPITCH + cb * ES;
          if constexpr (IS_I8) {
            int q[4];
#pragma unroll
            for (int e = 0; e < 4; ++e)
              q[e] = shift_round_clip<decltype(sat)::value>(acc[tn][tm][4 * g + e] + __builtin_bit_cast(int, m4[e]), a, qb);
            *reinterpret_cast<unsigned*>(dst) = pack_low_bytes(q[0], q[1], q[2], q[3]);
          } else {
            typedef float float2v __attribute__((ext_vector_type(2)));
            typedef _Float16 half2v __attribute__((ext_vector_type(2)));
            unsigned hw[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
              // rounded to fp32 before it is narrowed, and relu as a packed maximum on the narrowed pair: both as
              // in the unpooled kernel's epilogue
              float f0 = acc[tn][tm][4 * g + 2 * e] * m4[2 * e] + a4[2 * e];
              float f1 = acc[tn][tm][4 * g + 2 * e + 1] * m4[2 * e + 1] + a4[2 * e + 1];
              asm("" : "+v"(f0), "+v"(f1));   // (left alone the compiler merges the multiply-add and the narrowing into one instruction that rounds once)
              const float2v f = {f0, f1};
              half2v h = __builtin_convertvector(f, half2v);
              if (a.flags & F_RELU) h = __builtin_elementwise_max(h, half2v{(_Float16)0, (_Float16)0});
              hw[e] = __builtin_bit_cast(unsigned, h);
            }
            *reinterpret_cast<uint2*>(dst) = make_uint2(hw[0], hw[1]);
          }
        }
      }
    };
    if (!IS_I8 || qb.sat_ok) narrow(std::true_type{});
    else narrow(std::false_type{});
  }
  uint4* stg = ring + NW * XCH + wave * (32 * EP);
  constexpr int PPI = 64 / CG;  // pixels per pass of 64 lanes
  const int epix = lane / CG, ecg = lane % CG;
  const bool vec_ok = (a.K & 7) == 0;
  const OutLoc ol = EXT ? locate_output(a, ech) : OutLoc{nullptr, 0, 0};
  // All residual vectors of this lane first (tiles whose lanes finish at most 8 vectors: 32 registers), so
  // that they are in flight together behind the transpositions instead of one memory latency -- and one
  // wait for the previous store -- per stored vector.
  constexpr int ITS = 32 / PPI;
  constexpr bool PRE_RES = !POOL && TM_E * ITS <= 8;
  const bool pre_res = PRE_RES && (a.flags & F_RES) && vec_ok && !(EXT && nsplit > 1);
  uint4 resv[PRE_RES ? TM_E : 1][PRE_RES ? ITS : 1];
  if constexpr (PRE_RES) {
    if (pre_res) {
#pragma unroll
      for (int te = 0; te < TM_E; ++te)
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
          const int m = m0 + wm * WTM + (tm_lo + te) * 32 + it * PPI + epix;
          resv[te][it] = (m < a.M && ech < a.K) ? load_residual8<IS_I8>(a, m, ech) : make_uint4(0u, 0u, 0u, 0u);
        }
    }
  }
#pragma unroll
  for (int te = 0; te < (POOL ? 0 : TM_E); ++te) {
    const int tm = tm_lo + te;  // block row in the workgroup tile
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint4 v;
        if (SK == 2 && wk) {  // (wave-uniform) the upper half of the accumulator blocks
          v.x = as_u32(acc[tn][TM - TM_E + te][4 * g]);
          v.y = as_u32(acc[tn][TM - TM_E + te][4 * g + 1]);
          v.z = as_u32(acc[tn][TM - TM_E + te][4 * g + 2]);
          v.w = as_u32(acc[tn][TM - TM_E + te][4 * g + 3]);
        } else {
          v.x = as_u32(acc[tn][te][4 * g]);
          v.y = as_u32(acc[tn][te][4 * g + 1]);
          v.z = as_u32(acc[tn][te][4 * g + 2]);
          v.w = as_u32(acc[tn][te][4 * g + 3]);
        }
        stg[lrow * EP + tn * 8 + 2 * g + lhalf] = v;
      }
    // same wave wrote what it now reads: LDS operations of a wave execute in order
#pragma unroll
    for (int it = 0; it < 32 / PPI; ++it) {
      const int pix = it * PPI + epix;
      const uint4 lo = stg[pix * EP + ecg * 2], hi = stg[pix * EP + ecg * 2 + 1];
      const unsigned raw[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      const int m = m0 + wm * WTM + tm * 32 + pix;
      if (m >= a.M || ech >= a.K) continue;
      if (EXT && nsplit > 1) {  // (uniform) leave the raw partial sums for the workgroup that finishes the tile
        uint4* pp = reinterpret_cast<uint4*>(
            a.ws_part + ((size_t)(tile * nsplit + ks) * BM + (wm * WTM + tm * 32 + pix)) * BN + (ech - n0));
        pp[0] = lo;
        pp[1] = hi;
      } else {
        finish_store8<IS_I8, STOCH, EXT>(a, raw, m, ech, lp, ol, vec_ok, PRE_RES && pre_res, resv[PRE_RES ? te : 0][PRE_RES ? it : 0]);
      }
    }
  }
  if constexpr (POOL) {
    // ---- 3x3 / stride 2 / pad 1 max pool over the finished patch: pooled output (7 i + py, 8 j + px)
    //      takes conv outputs (2 oy - 1 + r, 2 ox - 1 + s), patch rows (2 py + r) * 17 + 2 px + s.
    __syncthreads();
    constexpr int GROUPS = BN / 8;
    const char* patch = reinterpret_cast<const char*>(ring);
    const int hp = a.Ho >> 1, wp = a.Wo >> 1;
    for (int item = tid; item < 56 * GROUPS; item += NW * 64) {
      const int pp = item / GROUPS, gch = item - pp * GROUPS;
      const int py = pp >> 3, px = pp & 7;
      const int oy = 7 * pool_i + py, ox = 8 * pool_j + px;
      const int ch = n0 + gch * 8;
      if (ch >= a.K) continue;
      // Only the first row and column of the image have a window that sticks out (2 oy - 1 < 0; the far
      // side ends at 2 oy + 1 <= Ho - 1): those read the centre row / column again instead, which
      // leaves the maximum as it is and the loop free of branches.
      const int r_lo = oy == 0 ? 1 : 0, s_lo = ox == 0 ? 1 : 0;
      typedef _Float16 half2v __attribute__((ext_vector_type(2)));
      typedef short short2v __attribute__((ext_vector_type(2)));
      uint4 best;
      unsigned ev[2], od[2];  // int8: the even and the odd bytes of a word as the high bytes of 16-bit lanes
#pragma unroll
      for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int s2 = 0; s2 < 3; ++s2) {
          const int rr = r == 0 ? r_lo : r, ss = s2 == 0 ? s_lo : s2;
          const char* src = patch + ((2 * py + rr) * PDX + 2 * px + ss) * PPITCH + gch * 8 * ES;  // 8-byte aligned
          uint4 v = make_uint4(0u, 0u, 0u, 0u);
          {
            const uint2 lo = *reinterpret_cast<const uint2*>(src);
            v.x = lo.x;
            v.y = lo.y;
            if constexpr (!IS_I8) {
              const uint2 hi = *reinterpret_cast<const uint2*>(src + 8);
              v.z = hi.x;
              v.w = hi.y;
            }
          }
          if constexpr (IS_I8) {
            const unsigned vw[2] = {v.x, v.y};
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              const unsigned e = (vw[h] << 8) & 0xff00ff00u, o = vw[h] & 0xff00ff00u;
              if (r == 0 && s2 == 0) {
                ev[h] = e;
                od[h] = o;
              } else {
                ev[h] = __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_bit_cast(short2v, ev[h]), __builtin_bit_cast(short2v, e)));
                od[h] = __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_bit_cast(short2v, od[h]), __builtin_bit_cast(short2v, o)));
              }
            }
          } else {
            if (r == 0 && s2 == 0) {
              best = v;
            } else {
              unsigned bw[4] = {best.x, best.y, best.z, best.w};
              const unsigned vw[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
              for (int h = 0; h < 4; ++h)
                bw[h] = __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_bit_cast(half2v, bw[h]), __builtin_bit_cast(half2v, vw[h])));
              best = make_uint4(bw[0], bw[1], bw[2], bw[3]);
            }
          }
        }
      if constexpr (IS_I8) best = make_uint4((ev[0] >> 8) | od[0], (ev[1] >> 8) | od[1], 0u, 0u);
      const size_t o = ((size_t)(pool_n * hp + oy) * wp + ox) * a.K + ch;
      if constexpr (IS_I8) *reinterpret_cast<uint2*>(static_cast<int8_t*>(a.y) + o) = make_uint2(best.x, best.y);
      else *reinterpret_cast<uint4*>(static_cast<_Float16*>(a.y) + o) = best;
    }
    return;
  }
  if (EXT && nsplit > 1) {
    // The workgroup that counts itself last owns the tile.  The XCDs' L2s are not coherent with
    // each other, so the partial tiles are released to device scope before the count (an L2
    // write-back) and acquired after it (an L2 invalidate).  One wave does that for the whole
    // workgroup, behind a barrier that has every wave's stores in L2: these fences act on the whole
    // L2, one per wave measured ~0.1 us per workgroup, serialised.  (Device-scope atomic stores and
    // loads for the partial sums themselves were far slower still.)  The winner leaves the counter
    // at zero for the next launch.  Nobody waits for anybody: the other workgroups are done once
    // they have counted.
    __shared__ int s_last;
    __syncthreads();
    if (tid == 0) {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      const unsigned old = atomicAdd(a.ws_cnt + tile * kCntStride, 1u);
      s_last = old == (unsigned)(nsplit - 1);
      if (s_last) {
        atomicExch(a.ws_cnt + tile * kCntStride, 0u);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      }
    }
    __syncthreads();
    if (!s_last) return;
    // A lane finishes NPOS positions of 1 pixel x 8 channels, one after another (this code must not
    // cost the main loop registers).  The partial tiles are added in split order, so the result does
    // not depend on who arrived when; JB of them are in flight at a time, because every load is a
    // round trip to memory (other XCDs wrote them).
    constexpr int NIT = 32 / PPI, NPOS = TM_E * NIT, JB = 8;
    typedef acc_t_scalar<IS_I8> sum_t;
    const unsigned* tile_part = a.ws_part + (size_t)tile * nsplit * BM * BN;
#pragma unroll 1
    for (int pos = 0; pos < NPOS; ++pos) {
      const int tm = tm_lo + pos / NIT, pix = (pos % NIT) * PPI + epix;
      const int m = m0 + wm * WTM + tm * 32 + pix;
      if (m >= a.M || ech >= a.K) continue;
      const unsigned* at = tile_part + (unsigned)((wm * WTM + tm * 32 + pix) * BN + (ech - n0));
      sum_t sum[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) sum[e] = 0;
#pragma unroll 1
      for (int j = 0; j < nsplit; j += JB) {
        uint4 lo[JB], hi[JB];
#pragma unroll
        for (int u = 0; u < JB; ++u) {
          const int jj = j + u < nsplit ? j + u : nsplit - 1;  // (uniform) past the end: a repeat that is not added
          const uint4* pp = reinterpret_cast<const uint4*>(at + (size_t)jj * BM * BN);
          lo[u] = pp[0];
          hi[u] = pp[1];
        }
#pragma unroll
        for (int u = 0; u < JB; ++u)
          if (j + u < nsplit) {
            const unsigned r[8] = {lo[u].x, lo[u].y, lo[u].z, lo[u].w, hi[u].x, hi[u].y, hi[u].z, hi[u].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) sum[e] += __builtin_bit_cast(sum_t, r[e]);
          }
      }
      unsigned raw[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) raw[e] = as_u32(sum[e]);
      finish_store8<IS_I8, STOCH, EXT>(a, raw, m, ech, lp, ol, vec_ok);
    }
  }
}

struct DmaTile {
  int waves_m, waves_n, tm, tn, ns, kp, sk;
  constexpr int bm() const { return waves_m * tm * 32; }
  constexpr int bn() const { return waves_n * tn * 32; }
};
// largest first; must match launch_typed
constexpr DmaTile kTiles[] = {
    {2, 2, 4, 2, 3, 1, 1},  // 256 x 128
    {4, 1, 4, 2, 3, 1, 1},  // 512 x 64
    {2, 1, 4, 2, 3, 1, 1},  // 256 x 64, two waves
    {2, 2, 2, 2, 3, 1, 1},  // 128 x 128
    {2, 2, 2, 1, 4, 1, 1},  // 128 x 64
    {2, 2, 1, 1, 4, 1, 1},  // 64 x 64
    // 128-byte chunks (need C % 64 == 0 for fp16, C % 128 == 0 for int8)
    {2, 2, 4, 2, 3, 2, 1},  // 256 x 128
    {2, 2, 4, 2, 2, 2, 1},  // 256 x 128, two stages
    {2, 2, 2, 2, 3, 2, 1},  // 128 x 128
    {2, 2, 2, 1, 3, 2, 1},  // 128 x 64
    {2, 2, 1, 1, 3, 2, 1},  // 64 x 64
    {2, 1, 4, 2, 3, 2, 1},  // 256 x 64, two waves
    // k-split wave pairs
    {2, 1, 2, 2, 3, 2, 2},  // 128 x 64, four waves of 64 x 64
    {1, 1, 2, 2, 3, 2, 2},  // 64 x 64, two waves of 64 x 64
    // tall tiles for layers with few output channels
    {4, 1, 2, 2, 3, 1, 1},  // 256 x 64, four waves of 64 x 64
    // 256-byte chunks: half as many barriers for the long reductions of the 512-channel layers
    {2, 2, 1, 1, 3, 4, 1},  // 64 x 64
    // short reductions over very many pixels (the first layer): a small ring, four workgroups per CU
    {2, 2, 2, 1, 3, 1, 1},  // 128 x 64
    // layers with at most 32 output channels over very many pixels (MobileNet's first layer): two waves, no
    // matrix work or epilogue lanes spent on channels that do not exist
    {2, 1, 2, 1, 3, 1, 1},  // 128 x 32
};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);

template <bool IS_I8, bool STOCH, int WAVES_M, int WAVES_N, int TM, int TN, int NS, int KP, int SK = 1>
hipError_t launch_one(const ConvArgs& a, hipStream_t st) {
  constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.K + BN - 1) / BN;
  const int tiles = tiles_m * tiles_n * (a.split > 1 ? a.split : 1);
  ConvArgs b = a;
  b.fd_tiles_m = make_fastdiv((uint32_t)tiles_m);
  b.fd_tiles_n = make_fastdiv((uint32_t)tiles_n);
  if (STOCH || a.nseg || a.split > 1)
    hipLaunchKernelGGL((igemm_dma_kernel<IS_I8, WAVES_M, WAVES_N, TM, TN, NS, KP, SK, STOCH, true>), dim3(tiles),
                       dim3(64 * WAVES_M * WAVES_N * SK), 0, st, b);
  else
    hipLaunchKernelGGL((igemm_dma_kernel<IS_I8, WAVES_M, WAVES_N, TM, TN, NS, KP, SK, false, false>), dim3(tiles),
                       dim3(64 * WAVES_M * WAVES_N * SK), 0, st, b);
  return hipGetLastError();
}

template <bool IS_I8, bool STOCH>
hipError_t launch_typed(const ConvArgs& a, int tile, hipStream_t st) {
  switch (tile) {
    case 0: return launch_one<IS_I8, STOCH, 2, 2, 4, 2, 3, 1>(a, st);
    case 1: return launch_one<IS_I8, STOCH, 4, 1, 4, 2, 3, 1>(a, st);
    case 2: return launch_one<IS_I8, STOCH, 2, 1, 4, 2, 3, 1>(a, st);
    case 3: return launch_one<IS_I8, STOCH, 2, 2, 2, 2, 3, 1>(a, st);
    case 4: return launch_one<IS_I8, STOCH, 2, 2, 2, 1, 4, 1>(a, st);
    case 5: return launch_one<IS_I8, STOCH, 2, 2, 1, 1, 4, 1>(a, st);
    case 6: return launch_one<IS_I8, STOCH, 2, 2, 4, 2, 3, 2>(a, st);
    case 7: return launch_one<IS_I8, STOCH, 2, 2, 4, 2, 2, 2>(a, st);
    case 8: return launch_one<IS_I8, STOCH, 2, 2, 2, 2, 3, 2>(a, st);
    case 9: return launch_one<IS_I8, STOCH, 2, 2, 2, 1, 3, 2>(a, st);
    case 10: return launch_one<IS_I8, STOCH, 2, 2, 1, 1, 3, 2>(a, st);
    case 11: return launch_one<IS_I8, STOCH, 2, 1, 4, 2, 3, 2>(a, st);
    case 12: return launch_one<IS_I8, STOCH, 2, 1, 2, 2, 3, 2, 2>(a, st);
    case 13: return launch_one<IS_I8, STOCH, 1, 1, 2, 2, 3, 2, 2>(a, st);
    case 14: return launch_one<IS_I8, STOCH, 4, 1, 2, 2, 3, 1, 1>(a, st);
    case 15: return launch_one<IS_I8, STOCH, 2, 2, 1, 1, 3, 4, 1>(a, st);
    case 16: return launch_one<IS_I8, STOCH, 2, 2, 2, 1, 3, 1, 1>(a, st);
    default: return launch_one<IS_I8, STOCH, 2, 1, 2, 1, 3, 1, 1>(a, st);
  }
}

long tiles_of(const ConvArgs& a, const DmaTile& t) {
  return (long)((a.M + t.bm() - 1) / t.bm()) * ((a.K + t.bn() - 1) / t.bn());
}

// can tile t run this layer?  (its chunk must divide the channel count)
bool tile_fits(const ConvArgs& a, bool is_i8, int t) {
  return t >= 0 && t < kNumTiles && a.C % (kTiles[t].kp * BKV * (is_i8 ? 16 : 8)) == 0;
}

// Tile choice from measured sweeps over the ResNet / MobileNet layer shapes: the 256x128
// tile once it gives every CU two workgroups, else 128x64, else 64x64 (small-M layers need
// the workgroup count more than the per-tile intensity); the longest chunks C and LDS allow.
int pick_tile(const ConvArgs& a, bool is_i8) {
  const bool kp2 = a.C % (2 * BKV * (is_i8 ? 16 : 8)) == 0;
  // short reductions over many pixels (the row-packed first layer, the early pointwise layers): a tile
  // lives for a handful of chunks, mostly the latency of its first loads and its stores; many
  // small-ring workgroups per CU overlap those
  // at most 32 output channels over very many pixels: the two-wave 128 x 32 tile (MobileNet's first layer at batch 32: 16.3 against 18.9 us)
  if (a.K <= 32 && a.Kred <= 8 * BKV * (is_i8 ? 16 : 8) && tiles_of(a, kTiles[17]) >= 1024) return 17;
  if (a.Kred <= 8 * BKV * (is_i8 ? 16 : 8) && tiles_of(a, kTiles[16]) >= 512) return 16;
  // 64 output channels over very many pixels in int8 (layer 1): tall tiles of 64 x 64 per wave
  if (a.K <= 64 && is_i8 && tiles_of(a, kTiles[14]) >= 384) return 14;
  if (a.K > 64 && tiles_of(a, kTiles[0]) >= 384) return 0;  // (measured down to 392 tiles: 737 vs 613 TFLOP/s on 512 -> 512 at 28 x 28)
  const int mid = kp2 ? 9 : 4;
  if (tiles_of(a, kTiles[mid]) >= 190) return mid;
  // a layer that gives each CU at most one 64 x 64 workgroup can afford the 96 KiB ring of 256-byte chunks
  if (a.C % (4 * BKV * (is_i8 ? 16 : 8)) == 0 && tiles_of(a, kTiles[15]) <= 256) return 15;
  return kp2 ? 10 : 5;
}

int resolve_tile(const ConvArgs& a, bool is_i8, int tile) {
  return tile_fits(a, is_i8, tile) ? tile : pick_tile(a, is_i8);
}

}  // namespace

bool igemm_dma_supported(const ConvArgs& a, bool is_i8) {
  const int es = is_i8 ? 1 : 2;
  const int ck = BKV * 16 / es;
  const size_t lim = 0x7fffffffu;  // buffer offsets are 32-bit and 0x80000000 marks "out of range"
  // tile rows are decoded as small offsets from the tile's first pixel (float reciprocal, < 2^22)
  return (a.C % ck) == 0 && a.R * a.S <= 32 && (size_t)a.N * a.xs_n * es <= lim &&
         (size_t)a.K * a.Kp * es <= lim && a.Wo < (1 << 20) && a.Ho < (1 << 20);
}

bool igemm_dma_pool_supported(const ConvArgs& a, bool is_i8) {
  // whole 7 x 8 blocks of pooled outputs, vector stores, the plain fused tail
  return igemm_dma_supported(a, is_i8) && a.Ho % 14 == 0 && a.Wo % 16 == 0 && (a.K & 7) == 0 && !(a.flags & F_RES) &&
         a.round_mode != ROUND_STOCHASTIC && a.nseg == 0;
}

void fill_pool_args(ConvArgs& a) {
  a.pool = 1;
  a.pool_tiles_row = (a.Wo / 2) / 8;
  a.pool_tiles_img = ((a.Ho / 2) / 7) * a.pool_tiles_row;
  a.fd_pool_row = make_fastdiv((uint32_t)a.pool_tiles_row);
  a.fd_pool_img = make_fastdiv((uint32_t)a.pool_tiles_img);
}

// 256 x 64 tiles of four 64 x 64 waves with a two-stage ring: 41 KB of LDS, three workgroups per CU.
// A workgroup's life is mostly latency (first loads, epilogue, pooling), so the third resident
// workgroup buys more than a third ring stage (measured on the 7x7 first layer of ResNet-18).
hipError_t launch_conv_igemm_dma_pool(const ConvArgs& a, bool is_i8, hipStream_t st) {
  constexpr int BN = 64;
  const int tiles_m = a.N * a.pool_tiles_img, tiles_n = (a.K + BN - 1) / BN;
  ConvArgs b = a;
  b.fd_tiles_m = make_fastdiv((uint32_t)tiles_m);
  b.fd_tiles_n = make_fastdiv((uint32_t)tiles_n);
  b.split = 1;
  if (is_i8)
    hipLaunchKernelGGL((igemm_dma_kernel<true, 4, 1, 2, 2, 2, 1, 1, false, false, true>), dim3(tiles_m * tiles_n), dim3(256), 0,
                       st, b);
  else
    hipLaunchKernelGGL((igemm_dma_kernel<false, 4, 1, 2, 2, 2, 1, 1, false, false, true>), dim3(tiles_m * tiles_n), dim3(256), 0,
                       st, b);
  return hipGetLastError();
}

void igemm_dma_pool_kernel_name(bool is_i8, char* buf, size_t len) {
  snprintf(buf, len, "igemm_dma_kernel<%s, 4, 1, 2, 2, 2, 1, 1, false, false, true>", is_i8 ? "true" : "false");
}

int igemm_dma_tile_count() { return kNumTiles; }

int igemm_dma_plan_split(const ConvArgs& a, bool is_i8, int tile, int want, size_t* counter_bytes,
                         size_t* total_bytes) {
  const DmaTile& t = kTiles[resolve_tile(a, is_i8, tile)];
  const int tiles = (int)tiles_of(a, t);
  const int chunks = a.Kred / (t.kp * BKV * (is_i8 ? 16 : 8));
  int split = want;
  if (split <= 0) {
    // Few tiles and a long reduction (the deep layers at small batch): the reduction is what can
    // still be spread over the idle CUs.  Handing a tile over costs about as much as six chunks of
    // the main loop and grows with the number of workgroups (measured on 7x7 and 14x14 layers of
    // 256 and 512 channels at batch 1 to 16): at least six chunks per workgroup, at most 128
    // workgroups, and only layers of at most 32 tiles and at least 24 chunks (int8: 12).
    split = 1;
    // (fp16, 18 chunks, 16 tiles -- 256 channels at 14 x 14, batch 1: 8.5 us unsplit, 9.3 us in three)
    if (tiles <= 32 && chunks >= (is_i8 ? 12 : 24)) {
      split = 128 / tiles;
      if (split > chunks / 6) split = chunks / 6;
      if (split > 16) split = 16;
    }
  }
  if (split > chunks) split = chunks;
  if (split < 1) split = 1;
  const int per = (chunks + split - 1) / split;
  split = (chunks + per - 1) / per;  // every workgroup gets at least one chunk
  *counter_bytes = (size_t)tiles * kCntStride * sizeof(unsigned);
  *total_bytes = split > 1 ? *counter_bytes + (size_t)tiles * split * t.bm() * t.bn() * 4 : 0;
  return split;
}

void igemm_dma_kernel_name(const ConvArgs& a, bool is_i8, int tile, char* buf, size_t len) {
  const DmaTile& t = kTiles[resolve_tile(a, is_i8, tile)];
  const bool stoch = is_i8 && a.round_mode == ROUND_STOCHASTIC;
  snprintf(buf, len, "igemm_dma_kernel<%s, %d, %d, %d, %d, %d, %d, %d, %s, %s, false>", is_i8 ? "true" : "false", t.waves_m,
           t.waves_n, t.tm, t.tn, t.ns, t.kp, t.sk, stoch ? "true" : "false",
           (stoch || a.nseg || a.split > 1) ? "true" : "false");
}

hipError_t launch_conv_igemm_dma(const ConvArgs& a, bool is_i8, int tile, hipStream_t st) {
  tile = resolve_tile(a, is_i8, tile);
  if (!is_i8) return launch_typed<false, false>(a, tile, st);
  return a.round_mode == ROUND_STOCHASTIC ? launch_typed<true, true>(a, tile, st) : launch_typed<true, false>(a, tile, st);
}

}  // namespace relay
