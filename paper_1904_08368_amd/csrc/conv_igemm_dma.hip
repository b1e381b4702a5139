// Implicit-GEMM conv2d for gfx950: MFMA main loop fed by direct global->LDS loads through a
// multi-stage LDS ring, fused epilogue in registers (paper Section 4.1 / 4.2).
//
// GEMM view: rows m = (image, p, q) output pixels, columns = output channels, reduction
// kk = (r, s, c).  NHWC activations and [k][r][s][c] filters are both contiguous along the
// reduction axis and move as 16-byte k-vectors.  A workgroup owns BM pixels x BN channels;
// a wave owns TM x TN MFMA blocks of 32x32 (filters are the A operand, so a lane ends up
// with 4 consecutive channels of one pixel per accumulator group = one NHWC store).
//
// Staging: per 64-byte reduction chunk every wave issues `buffer_load_dwordx4 ... lds`
// instructions, each moving 16 tile rows x 64 B straight into LDS (lane i writes 16 bytes
// at base + 16*i), no VGPRs involved.  The LDS bank swizzle is applied on the global side:
// lane i fetches the k-vector that belongs in its fixed LDS slot.  Filter taps that fall in
// the padding, rows past the end of the tensor and channels past Cout are given a buffer
// offset beyond num_records; the buffer unit then writes zeros (checked on hardware), so
// the MFMA loop has no special cases.  NS ring stages keep NS-1 chunks in flight behind one
// barrier per chunk.  The loads are inline asm on purpose: the compiler, not seeing LDS
// written, does not drain the memory pipeline before every LDS read; ordering is by the
// explicit vmcnt waits and barriers below.
//
// Needs C to be a whole number of chunks (32 halves / 64 int8) and R*S <= 32; other shapes
// go to the register-staged kernel in conv_igemm.hip.
#include <cstdio>

#include "igemm_common.hpp"

namespace relay {
namespace {

__device__ __forceinline__ void lds_dma16(intx4 rsrc, unsigned lds_base, unsigned voff) {
  // m0 = wave-uniform LDS byte address; lane i lands at m0 + 16*i
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds_base), "v"(voff),
               "s"(rsrc)
               : "memory");
}

// Wait until at most N of this wave's global->LDS loads are pending and all of its LDS reads
// have returned (so that the stage they read may be refilled after the barrier).
template <int N>
__device__ __forceinline__ void wait_loads() {
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(N) : "memory");
}

__device__ __forceinline__ intx4 make_rsrc(const void* p, unsigned bytes) {
  const unsigned long long pa = reinterpret_cast<unsigned long long>(p);
  intx4 r;
  r[0] = (int)(unsigned)pa;
  r[1] = (int)(unsigned)((pa >> 32) & 0xffffu);  // stride 0: raw buffer
  r[2] = (int)bytes;                            // num_records
  r[3] = 0x00020000;                            // 32-bit data format, no swizzle
  return r;
}

constexpr unsigned kOob = 0x80000000u;  // beyond any num_records this library accepts

template <bool IS_I8, int WAVES_M, int WAVES_N, int TM, int TN, int NS>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, 2) void igemm_dma_kernel(const ConvArgs a) {
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int VE = IS_I8 ? 16 : 8;
  constexpr int ES = IS_I8 ? 1 : 2;
  constexpr int CK = BKV * VE;
  constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
  constexpr int WTM = TM * 32, WTN = TN * 32;
  constexpr int XB = BM / 16, WB = BN / 16;  // 1 KiB staging blocks: 16 rows x 64 B
  static_assert(XB % NW == 0 && WB % NW == 0, "staging blocks must divide over the waves");
  constexpr int XL = XB / NW, WL = WB / NW, LPC = XL + WL;  // loads per chunk per wave
  constexpr int STAGE = (BM + BN) * BKV;                    // 16-byte slots per ring stage
  static_assert((NS - 1) * LPC <= 63, "vmcnt is a 6-bit counter");
  typedef typename Mma<IS_I8>::acc_t acc_t;
  typedef typename Mma<IS_I8>::scalar_t scalar_t;

  __shared__ uint4 ring[NS * STAGE];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.K + BN - 1) / BN;
  const int tile = xcd_remap(blockIdx.x, tiles_m * tiles_n);
  const int tile_n = tile % tiles_n, tile_m = tile / tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // ---- staging role of this lane inside a 16-row block: row srow, physical slot sphys
  const int srow = lane >> 2, sphys = lane & 3;
  int x_off[XL];        // byte offset of tap (0,0), channel 0 of the row's k-vector
  unsigned x_taps[XL];  // bit t set: tap t of this row lies inside the image
  const int HoWo = a.Ho * a.Wo;
#pragma unroll
  for (int j = 0; j < XL; ++j) {
    const int row = (wave * XL + j) * 16 + srow;
    const int kvl = sphys ^ ((row >> 1) & (BKV - 1));
    const int m = m0 + row;
    unsigned taps = 0;
    int off = 0;
    if (m < a.M) {
      const int n = m / HoWo;
      const int rem = m - n * HoWo;
      const int p = rem / a.Wo;
      const int q = rem - p * a.Wo;
      const int ih0 = p * a.sh - a.ph, iw0 = q * a.sw - a.pw;
      off = (((n * a.H + ih0) * a.W + iw0) * a.C + kvl * VE) * ES;
      int t = 0;
      for (int r = 0; r < a.R; ++r)
        for (int s = 0; s < a.S; ++s, ++t)
          if ((unsigned)(ih0 + r) < (unsigned)a.H && (unsigned)(iw0 + s) < (unsigned)a.W) taps |= 1u << t;
    }
    x_off[j] = off;
    x_taps[j] = taps;
  }
  unsigned w_off[WL];
#pragma unroll
  for (int j = 0; j < WL; ++j) {
    const int row = (wave * WL + j) * 16 + srow;
    const int kvl = sphys ^ ((row >> 1) & (BKV - 1));
    const int ch = n0 + row;
    w_off[j] = ch < a.K ? (unsigned)((ch * a.Kp + kvl * VE) * ES) : kOob;
  }
  const intx4 rs_x = make_rsrc(a.x, (unsigned)((size_t)a.N * a.H * a.W * a.C * ES));
  const intx4 rs_w = make_rsrc(a.w, (unsigned)((size_t)a.K * a.Kp * ES));
  const unsigned ring_base = (unsigned)(size_t)(__attribute__((address_space(3))) uint4*)(&ring[0]);

  // reduction position of the next chunk to be issued (wave-uniform)
  int is_tap = 0, is_r = 0, is_s = 0, is_c = 0, is_kc = 0;
  auto issue_chunk = [&](int stage) {
    const unsigned delta = (unsigned)(((is_r * a.W + is_s) * a.C + is_c) * ES);
    const unsigned sbase = ring_base + (unsigned)(stage * STAGE) * 16u;
#pragma unroll
    for (int j = 0; j < XL; ++j) {
      const unsigned voff = ((x_taps[j] >> is_tap) & 1u) ? (unsigned)x_off[j] + delta : kOob;
      lds_dma16(rs_x, sbase + (unsigned)((wave * XL + j) * 64) * 16u, voff);
    }
    const unsigned wdelta = (unsigned)(is_kc * CK * ES);
#pragma unroll
    for (int j = 0; j < WL; ++j)
      lds_dma16(rs_w, sbase + (unsigned)(BM * BKV + (wave * WL + j) * 64) * 16u, w_off[j] + wdelta);
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
  };

  acc_t acc[TN][TM];
#pragma unroll
  for (int tn = 0; tn < TN; ++tn)
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tn][tm][v] = 0;

  const int nchunks = a.Kred / CK;
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (s < nchunks) issue_chunk(s);

  const int lrow = lane & 31, lhalf = lane >> 5;
  int stage = 0;           // ring stage of chunk kc
  int fill = NS - 1;       // ring stage the next issued chunk goes to
  for (int kc = 0; kc < nchunks; ++kc) {
    // chunk kc has landed once at most the loads of the chunks issued after it are pending
    if (kc + NS - 2 < nchunks)
      wait_loads<(NS - 2) * LPC>();
    else
      wait_loads<0>();
    __builtin_amdgcn_s_barrier();  // everyone's part of chunk kc is in LDS; stage `fill` is free again
    if (kc + NS - 1 < nchunks) issue_chunk(fill);
    const uint4* xs = ring + stage * STAGE;
    const uint4* ws = xs + BM * BKV;
#pragma unroll
    for (int ks = 0; ks < BKV / 2; ++ks) {
      const int kq = 2 * ks + lhalf;
      uint4 wf[TN], xf[TM];
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) wf[tn] = ws[lds_slot(wn * WTN + tn * 32 + lrow, kq)];
#pragma unroll
      for (int tm = 0; tm < TM; ++tm) xf[tm] = xs[lds_slot(wm * WTM + tm * 32 + lrow, kq)];
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = Mma<IS_I8>::mma(wf[tn], xf[tm], acc[tn][tm]);
    }
    stage = stage + 1 == NS ? 0 : stage + 1;
    fill = fill + 1 == NS ? 0 : fill + 1;
  }

  // ---- epilogue: element v of a 32x32 accumulator block is channel 8*(v/4) + 4*(lane/32) + v%4
  //      of pixel lane%32.  Per-channel constants are fetched before any store.
  const bool vec_ok = (a.K & 3) == 0;
#pragma unroll
  for (int tn = 0; tn < TN; ++tn) {
    EpiParams ep[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) ep[g] = load_epi_params<IS_I8>(a, n0 + wn * WTN + tn * 32 + 8 * g + 4 * lhalf);
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
      const int m = m0 + wm * WTM + tm * 32 + lrow;
      if (m >= a.M) continue;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int ch = n0 + wn * WTN + tn * 32 + 8 * g + 4 * lhalf;
        if (ch >= a.K) continue;
        const scalar_t v[4] = {acc[tn][tm][4 * g], acc[tn][tm][4 * g + 1], acc[tn][tm][4 * g + 2],
                               acc[tn][tm][4 * g + 3]};
        epilogue_store4<IS_I8>(a, v, m, ch, ep[g], vec_ok);
      }
    }
  }
}

struct DmaTile {
  int waves_m, waves_n, tm, tn, ns;
  constexpr int bm() const { return waves_m * tm * 32; }
  constexpr int bn() const { return waves_n * tn * 32; }
};
// largest first; must match launch_typed
constexpr DmaTile kTiles[] = {
    {2, 2, 4, 2, 3},  // 256 x 128
    {4, 1, 4, 2, 3},  // 512 x 64
    {2, 1, 4, 2, 3},  // 256 x 64, two waves
    {2, 2, 2, 2, 3},  // 128 x 128
    {2, 2, 2, 1, 4},  // 128 x 64
    {2, 2, 1, 1, 4},  // 64 x 64
};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);

template <bool IS_I8, int WAVES_M, int WAVES_N, int TM, int TN, int NS>
hipError_t launch_one(const ConvArgs& a, hipStream_t st) {
  constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
  const int tiles = ((a.M + BM - 1) / BM) * ((a.K + BN - 1) / BN);
  hipLaunchKernelGGL((igemm_dma_kernel<IS_I8, WAVES_M, WAVES_N, TM, TN, NS>), dim3(tiles), dim3(64 * WAVES_M * WAVES_N),
                     0, st, a);
  return hipGetLastError();
}

template <bool IS_I8>
hipError_t launch_typed(const ConvArgs& a, int tile, hipStream_t st) {
  switch (tile) {
    case 0: return launch_one<IS_I8, 2, 2, 4, 2, 3>(a, st);
    case 1: return launch_one<IS_I8, 4, 1, 4, 2, 3>(a, st);
    case 2: return launch_one<IS_I8, 2, 1, 4, 2, 3>(a, st);
    case 3: return launch_one<IS_I8, 2, 2, 2, 2, 3>(a, st);
    case 4: return launch_one<IS_I8, 2, 2, 2, 1, 4>(a, st);
    default: return launch_one<IS_I8, 2, 2, 1, 1, 4>(a, st);
  }
}

long tiles_of(const ConvArgs& a, const DmaTile& t) {
  return (long)((a.M + t.bm() - 1) / t.bm()) * ((a.K + t.bn() - 1) / t.bn());
}

// Largest tile that still gives every compute unit a workgroup; smaller tiles as the layer shrinks.
int pick_tile(const ConvArgs& a) {
  for (int t = 0; t < kNumTiles; ++t) {
    if (kTiles[t].bn() > 64 && a.K <= 64) continue;
    if (tiles_of(a, kTiles[t]) >= 256) return t;
  }
  return kNumTiles - 1;
}

}  // namespace

bool igemm_dma_supported(const ConvArgs& a, bool is_i8) {
  const int es = is_i8 ? 1 : 2;
  const int ck = BKV * 16 / es;
  const size_t lim = 0x7fffffffu;  // buffer offsets are 32-bit and 0x80000000 marks "out of range"
  return (a.C % ck) == 0 && a.R * a.S <= 32 && (size_t)a.N * a.H * a.W * a.C * es <= lim &&
         (size_t)a.K * a.Kp * es <= lim;
}

int igemm_dma_tile_count() { return kNumTiles; }

void igemm_dma_kernel_name(const ConvArgs& a, bool is_i8, int tile, char* buf, size_t len) {
  if (tile < 0 || tile >= kNumTiles) tile = pick_tile(a);
  const DmaTile& t = kTiles[tile];
  snprintf(buf, len, "igemm_dma_kernel<%s, %d, %d, %d, %d, %d>", is_i8 ? "true" : "false", t.waves_m, t.waves_n, t.tm,
           t.tn, t.ns);
}

hipError_t launch_conv_igemm_dma(const ConvArgs& a, bool is_i8, int tile, hipStream_t st) {
  if (tile < 0 || tile >= kNumTiles) tile = pick_tile(a);
  return is_i8 ? launch_typed<true>(a, tile, st) : launch_typed<false>(a, tile, st);
}

}  // namespace relay
