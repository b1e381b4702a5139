// Implicit-GEMM conv2d on gfx950 MFMA with the fused epilogue in registers.
//
// One fused primitive function (paper Section 4.1): conv2d followed by the elementwise
// operators that fusion folds behind it.  fp16 x fp16 -> fp32 (v_mfma_f32_32x32x16_f16)
// and int8 x int8 -> int32 (v_mfma_i32_32x32x32_i8), the latter with the realized
// quantize operator of Section 4.2 as epilogue.
//
// GEMM view: rows m = (image, p, q) output pixels, columns = output channels, reduction
// index kk = (r, s, c).  Activations are NHWC and filters [k][r][s][c], so both operands
// are contiguous along the reduction axis and move as 16-byte "k-vectors" (8 halves or
// 16 int8).  Filters are the MFMA A operand (rows of the accumulator block = channels):
// a lane then owns 4 consecutive channels of one pixel per accumulator group, which is
// one 8-byte (fp16) or 4-byte (int8) NHWC store.
//
// A workgroup owns a BM-pixel x BN-channel tile.  Per 64-byte reduction chunk it stages
// BM+BN rows through LDS (double buffered, one barrier per chunk); global loads of chunk
// i+1 are in flight while the MFMAs of chunk i run.  Padding taps and ragged rows are
// loaded as zeros, so the main loop has no special cases.
#include <cstdio>

#include "igemm_common.hpp"

namespace relay {
namespace {

template <bool IS_I8, int BM, int BN, int WAVES_M, int WAVES_N, bool FAST>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void igemm_conv_kernel(const ConvArgs a) {
  constexpr int NT = 64 * WAVES_M * WAVES_N;
  constexpr int VE = IS_I8 ? 16 : 8;  // elements per k-vector
  constexpr int ES = IS_I8 ? 1 : 2;   // bytes per element
  constexpr int CK = BKV * VE;        // reduction elements per chunk
  constexpr int WTM = BM / WAVES_M, WTN = BN / WAVES_N;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int XL = BM * BKV / NT, WL = BN * BKV / NT;
  constexpr int ROWS_PER_PASS = NT / BKV;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be whole 32x32 blocks");
  static_assert((BM * BKV) % NT == 0 && (BN * BKV) % NT == 0, "staging must divide evenly");
  typedef typename Mma<IS_I8>::acc_t acc_t;
  typedef typename Mma<IS_I8>::scalar_t scalar_t;

  __shared__ uint4 lds[2][(BM + BN) * BKV];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  const int tiles_m = (a.M + BM - 1) / BM;
  const int tile_m = blockIdx.x % tiles_m, tile_n = blockIdx.x / tiles_m;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // ---- staging roles: this thread moves k-vector `kv` of rows row0 + i*ROWS_PER_PASS
  const int kv = tid % BKV;
  const int row0 = tid / BKV;
  int x_ih0[XL], x_iw0[XL], x_base[XL];
  const int HoWo = a.Ho * a.Wo;
#pragma unroll
  for (int i = 0; i < XL; ++i) {
    const int m = m0 + row0 + i * ROWS_PER_PASS;
    if (m < a.M) {
      const int n = m / HoWo;
      const int rem = m - n * HoWo;
      const int p = rem / a.Wo;
      const int q = rem - p * a.Wo;
      x_ih0[i] = p * a.sh - a.ph;
      x_iw0[i] = q * a.sw - a.pw;
      x_base[i] = n * a.H * a.W * a.C;
    } else {
      x_ih0[i] = -(1 << 30);  // every tap of a ragged row tests out of range
      x_iw0[i] = 0;
      x_base[i] = 0;
    }
  }
  const char* xb = static_cast<const char*>(a.x);
  const char* wb = static_cast<const char*>(a.w);
  const uint4 zero4 = make_uint4(0, 0, 0, 0);

  uint4 xr[XL], wr[WL];
  // FAST: C is a whole number of chunks, so a chunk lies inside one filter tap (r, s).
  int tap_r = 0, tap_s = 0, tap_c = 0;
  auto load_chunk = [&](int kc) {
    int r, s, c;
    bool kok = true;
    if (FAST) {
      r = tap_r;
      s = tap_s;
      c = tap_c + kv * VE;
    } else {
      const int kk = kc * CK + kv * VE;  // a k-vector never straddles a tap (C % VE == 0)
      const int tap = kk / a.C;
      c = kk - tap * a.C;
      r = tap / a.S;
      s = tap - r * a.S;
      kok = kk < a.Kred;
    }
#pragma unroll
    for (int i = 0; i < XL; ++i) {
      const int ih = x_ih0[i] + r, iw = x_iw0[i] + s;
      const bool ok = kok && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
      const long off = ((long)x_base[i] + ((long)ih * a.W + iw) * a.C + c) * ES;
      xr[i] = ok ? *reinterpret_cast<const uint4*>(xb + off) : zero4;
    }
#pragma unroll
    for (int i = 0; i < WL; ++i) {
      const int row = n0 + row0 + i * ROWS_PER_PASS;
      const size_t off = ((size_t)row * a.Kp + (size_t)kc * CK + kv * VE) * ES;
      wr[i] = (row < a.K) ? *reinterpret_cast<const uint4*>(wb + off) : zero4;
    }
    if (FAST) {
      tap_c += CK;
      if (tap_c == a.C) {
        tap_c = 0;
        if (++tap_s == a.S) {
          tap_s = 0;
          ++tap_r;
        }
      }
    }
  };
  auto store_chunk = [&](int buf) {
#pragma unroll
    for (int i = 0; i < XL; ++i) {
      const int row = row0 + i * ROWS_PER_PASS;
      lds[buf][lds_slot(row, kv)] = xr[i];
    }
#pragma unroll
    for (int i = 0; i < WL; ++i) {
      const int row = row0 + i * ROWS_PER_PASS;
      lds[buf][BM * BKV + lds_slot(row, kv)] = wr[i];
    }
  };

  acc_t acc[TN][TM];
#pragma unroll
  for (int tn = 0; tn < TN; ++tn)
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tn][tm][v] = 0;

  const int nchunks = (a.Kred + CK - 1) / CK;
  load_chunk(0);
  store_chunk(0);
  __syncthreads();

  const int lrow = lane & 31, lhalf = lane >> 5;
  for (int kc = 0; kc < nchunks; ++kc) {
    const int buf = kc & 1;
    if (kc + 1 < nchunks) load_chunk(kc + 1);
#pragma unroll
    for (int ks = 0; ks < BKV / 2; ++ks) {
      const int kq = 2 * ks + lhalf;
      uint4 wf[TN], xf[TM];
#pragma unroll
      for (int tn = 0; tn < TN; ++tn) wf[tn] = lds[buf][BM * BKV + lds_slot(wn * WTN + tn * 32 + lrow, kq)];
#pragma unroll
      for (int tm = 0; tm < TM; ++tm) xf[tm] = lds[buf][lds_slot(wm * WTM + tm * 32 + lrow, kq)];
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = Mma<IS_I8>::mma(wf[tn], xf[tm], acc[tn][tm]);
    }
    if (kc + 1 < nchunks) store_chunk(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: accumulator element v of a 32x32 block is channel 8*(v/4) + 4*(lane/32) + v%4
  //      (block row) of pixel lane%32 (block column).
  const bool vec_ok = (a.K & 3) == 0;
  EpiParams ep[TN][4];
#pragma unroll
  for (int tn = 0; tn < TN; ++tn)
#pragma unroll
    for (int g = 0; g < 4; ++g) ep[tn][g] = load_epi_params<IS_I8>(a, n0 + wn * WTN + tn * 32 + 8 * g + 4 * lhalf);
#pragma unroll
  for (int tm = 0; tm < TM; ++tm) {
    const int m = m0 + wm * WTM + tm * 32 + lrow;
    if (m >= a.M) continue;
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int ch = n0 + wn * WTN + tn * 32 + 8 * g + 4 * lhalf;
        if (ch >= a.K) continue;
        const scalar_t v[4] = {acc[tn][tm][4 * g], acc[tn][tm][4 * g + 1], acc[tn][tm][4 * g + 2],
                               acc[tn][tm][4 * g + 3]};
        epilogue_store4<IS_I8>(a, v, m, ch, ep[tn][g], vec_ok);
      }
  }
}

struct TileShape {
  int bm, bn, waves_m, waves_n;
};
// tile ids, largest first (must match launch_typed)
constexpr TileShape kTiles[] = {{256, 128, 2, 2}, {256, 64, 4, 1}, {128, 128, 2, 2}, {128, 64, 2, 2}, {64, 64, 2, 2}};
constexpr int kNumTiles = sizeof(kTiles) / sizeof(kTiles[0]);

template <bool IS_I8, int BM, int BN, int WAVES_M, int WAVES_N>
hipError_t launch_one(const ConvArgs& a, bool fast, hipStream_t st) {
  const int tiles = ((a.M + BM - 1) / BM) * ((a.K + BN - 1) / BN);
  dim3 grid(tiles), block(64 * WAVES_M * WAVES_N);
  if (fast)
    hipLaunchKernelGGL((igemm_conv_kernel<IS_I8, BM, BN, WAVES_M, WAVES_N, true>), grid, block, 0, st, a);
  else
    hipLaunchKernelGGL((igemm_conv_kernel<IS_I8, BM, BN, WAVES_M, WAVES_N, false>), grid, block, 0, st, a);
  return hipGetLastError();
}

template <bool IS_I8>
hipError_t launch_typed(const ConvArgs& a, int tile, bool fast, hipStream_t st) {
  switch (tile) {
    case 0: return launch_one<IS_I8, 256, 128, 2, 2>(a, fast, st);
    case 1: return launch_one<IS_I8, 256, 64, 4, 1>(a, fast, st);
    case 2: return launch_one<IS_I8, 128, 128, 2, 2>(a, fast, st);
    case 3: return launch_one<IS_I8, 128, 64, 2, 2>(a, fast, st);
    default: return launch_one<IS_I8, 64, 64, 2, 2>(a, fast, st);
  }
}

// Largest tile that still gives every compute unit work; smaller tiles as the layer shrinks.
int pick_tile(const ConvArgs& a) {
  const long want = 256;  // compute units
  for (int t = 0; t < kNumTiles; ++t) {
    if (kTiles[t].bn > 64 && a.K <= 64) continue;
    const long tiles = (long)((a.M + kTiles[t].bm - 1) / kTiles[t].bm) * ((a.K + kTiles[t].bn - 1) / kTiles[t].bn);
    if (tiles >= want) return t;
  }
  return kNumTiles - 1;
}

}  // namespace

int igemm_tile_count() { return kNumTiles; }

void igemm_kernel_name(const ConvArgs& a, bool is_i8, int tile, char* buf, size_t len) {
  if (tile < 0 || tile >= kNumTiles) tile = pick_tile(a);
  const bool fast = (a.C % (BKV * (is_i8 ? 16 : 8))) == 0;
  snprintf(buf, len, "igemm_conv_kernel<%s, %d, %d, %d, %d, %s>", is_i8 ? "true" : "false", kTiles[tile].bm,
           kTiles[tile].bn, kTiles[tile].waves_m, kTiles[tile].waves_n, fast ? "true" : "false");
}

hipError_t launch_conv_igemm(const ConvArgs& a, bool is_i8, int tile, hipStream_t st) {
  const int ck = BKV * (is_i8 ? 16 : 8);
  const bool fast = (a.C % ck) == 0;
  if (tile < 0 || tile >= kNumTiles) tile = pick_tile(a);
  return is_i8 ? launch_typed<true>(a, tile, fast, st) : launch_typed<false>(a, tile, fast, st);
}

}  // namespace relay
