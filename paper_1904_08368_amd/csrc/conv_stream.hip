// 3x3 / stride 1 / pad 1 conv2d for gfx950 as a PERSISTENT workgroup that streams tile after tile
// (paper Section 4.1 / 4.2: the same fused primitive function as conv_igemm_dma.hip and
// conv_halo.hip; another schedule).
//
// Why: on the layers of the vision workloads a workgroup of the one-tile-per-workgroup kernels
// lives for ~12 k clocks of which the matrix cores work ~2.3 k: the rest is the serial chain
// argument fetch -> address decoding -> first loads -> memory latency -> reduction -> transposition
// -> stores, paid once per tile, and a layer whose tile count is 1.6 times the number of resident
// workgroups pays it twice.  Here a workgroup is launched once per compute unit and walks a list
// of tiles; the global->LDS loads of the next tile (activations and filters) are issued from inside
// the current tile's reduction, the next tile's reduction starts in the same loop iteration in
// which the current tile's last products are formed, and the stores of a finished tile drain under
// the following reduction.  Per tile only the epilogue arithmetic is not overlapped.
//
// Coordinates as in conv_halo.hip: pixels are numbered o = n*F + p*P + q with P = W + 1 and
// F = (H + 1)*P, so that filter tap (r, s) is the constant shift r*P + s and one staged run of
// BM + 2P + 2 input positions (the halo) serves all nine taps.  A "unit" is one (tile, chunk of CK
// input channels); its halo is loaded once into one of two LDS buffers while the previous unit is
// being reduced.  Filters go through a three-stage ring, one (tap, chunk) slab per stage.
//
// Loop shape.  A step is one (unit, tap).  Every wave issues, behind the matrix instructions of a
// step, the same number L of global->LDS loads: its share of the filters of the step after next
// and of the next unit's halo (loads that do not exist go, out of range, to a dump block), so the
// waits are compile-time counts.  The second half of a step's matrix instructions is carried
// across the barrier of the next step and runs while that step's first operands come out of LDS.
// The epilogue works on the accumulators where they are (element v of a 32x32 block: pixel
// lane % 32, channels 8 (v / 4) + 4 (lane / 32) + v % 4): per-channel constants from an LDS table,
// residual and result as 8-byte (fp16) or 4-byte (int8) pieces through buffer descriptors whose
// out-of-range offsets read zeros / drop the store, so that every tile issues the same number of
// memory instructions whatever its shape.
//
// vmcnt bookkeeping (memory instructions of a wave complete in issue order on this chip; loads and
// stores share the counter).  The residual loads are inline asm like the global->LDS loads: a load
// the compiler knows about makes it insert waits that count only what it knows, and those stall on
// the ring loads just issued.  Every unit issues R residual loads in front of its tap 6 (real ones
// in a tile's last unit, out-of-range fillers before); the wait of tap 8 (at most L younger
// instructions pending) has them landed, two steps later, and only then are the registers handed
// to the compiler as values.  Issue order around the end of a tile whose last step is g:
//   slot(g-3) | R residual loads | slot(g-2) | slot(g-1) | slot(g) | slot(g+1) | S stores | slot(g+2) ...
// step g-2 needs slot(g-4): at most L + R younger instructions may be pending; step g-1 needs
// slot(g-3): L + R; steps g and g+1: L; step g+2 needs slot(g): L + S; step g+3 needs slot(g+1):
// S + L; from step g+4 on L again.
#include <cstdio>

#include <atomic>
#include <type_traits>

#include "dma_common.hpp"

namespace relay {
namespace {

struct StreamGeom {
  int P, F, Mflat;
  int xblk;                 // 16-row blocks per 64-byte plane of a halo buffer
  int ncc;                  // channel chunks per tile, C / CK
  int tiles_m, tiles_n;     // tiles of BM flat positions / BN channels
  int gm;                   // workgroups along the position axis: workgroup (bn, bm) walks tile_m = bm, bm + gm, ...
  FastDiv fd_f, fd_p, fd_xblk, fd_tiles_n;
};

// FA = how many steps ahead of its use a filter slab is fetched (ring of FA + 1 stages).  Memory
// instructions complete in issue order, so the wait of step g -- "everything up to the slot that
// fetched this step's filters has landed" -- also forces every older load: a load issued in slot g has
// FA steps to land, whatever it is.  The activations come from HBM (several thousand clocks under
// load, a step is ~500): FA = 2 makes every step wait for them.  The next unit's halo is therefore
// issued in the first 10 - FA slots of a unit, the residual loads in front of slot 9 - FA: the wait
// of the next unit's first step is then the first that needs them and has them.
constexpr int ring_stages(int fa) { return fa + 1; }
constexpr int halo_slots(int fa) { return 10 - fa; }

typedef _Float16 half4v __attribute__((ext_vector_type(4)));
typedef unsigned uintx2 __attribute__((ext_vector_type(2)));

template <bool IS_I8, int WAVES_M, int WAVES_N, int TM, int TN, int KP, int HB, int WGS, int FA>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, WGS) void conv3x3_stream_kernel(const ConvArgs a, const StreamGeom g) {
  constexpr int NSW = ring_stages(FA), XS = halo_slots(FA);
  static_assert(FA >= 2 && FA <= 7, "the look-ahead wraps at most once into the next unit");
  constexpr int NW = WAVES_M * WAVES_N;
  constexpr int VE = IS_I8 ? 16 : 8;
  constexpr int ES = IS_I8 ? 1 : 2;
  constexpr int CK = KP * BKV * VE;
  constexpr int BM = WAVES_M * TM * 32, BN = WAVES_N * TN * 32;
  constexpr int WTM = TM * 32, WTN = TN * 32;
  constexpr int FB = KP * (BN / 16);       // 16-row filter blocks per step
  static_assert(FB % NW == 0 || NW % FB == 0, "filter blocks must divide over the waves");
  constexpr int LW = FB >= NW ? FB / NW : 1;   // filter loads per step per wave (fewer blocks than waves: the others issue fillers)
  constexpr int L = LW + HB;               // loads per step per wave
  constexpr int KSTEPS = KP * (BKV / 2);
  constexpr int HK = KSTEPS / 2;           // k-steps whose products are formed in the step's own iteration
  constexpr int DK = KSTEPS - HK;          // ... carried into the next iteration
  constexpr int NRES = TM * TN * 4;        // residual loads and stores of a tile, per lane
  constexpr int WBASE = (FA - 1) * L;      // younger loads that may be pending at a step's wait
  static_assert(WBASE + 2 * NRES <= 63, "vmcnt is a 6-bit counter");
  constexpr int WPLANE = BN * BKV;         // 16-byte slots of one filter plane
  constexpr int WSTAGE = KP * WPLANE;
  typedef typename Mma<IS_I8>::acc_t acc_t;

  extern __shared__ uint4 lds[];
  const int xplane = g.xblk * 64;          // slots of one halo plane
  const int xbuf_slots = KP * xplane;
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) uint4*)(&lds[0]);
  const unsigned wring_base = lds_base + (unsigned)(2 * xbuf_slots) * 16u;
  const unsigned dump_base = wring_base + (unsigned)(NSW * WSTAGE) * 16u;
  const uint4* wring = lds + 2 * xbuf_slots;
  float* cst = reinterpret_cast<float*>(lds + 2 * xbuf_slots + NSW * WSTAGE + 64);   // [2][BN]: mul, add (int8: bias bits)

  asm volatile("" ::"s"(a.x), "s"(a.w), "s"(a.y), "s"(a.res), "s"(a.bias), "s"(a.scale), "s"(a.shift), "s"(a.qbias));
  asm volatile("" ::"s"(a.N), "s"(a.H), "s"(a.W), "s"(a.C), "s"(a.K), "s"(a.Kp), "s"(a.flags), "s"(a.xs_n), "s"(a.M));
  asm volatile("" ::"s"(g.P), "s"(g.F), "s"(g.Mflat), "s"(g.xblk), "s"(g.ncc), "s"(g.tiles_m), "s"(g.tiles_n), "s"(g.gm),
               "s"(g.fd_f.mul), "s"(g.fd_f.shift), "s"(g.fd_p.mul), "s"(g.fd_p.shift), "s"(g.fd_xblk.mul), "s"(g.fd_xblk.shift),
               "s"(g.fd_tiles_n.mul), "s"(g.fd_tiles_n.shift));
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  const int lid = xcd_remap(blockIdx.x, gridDim.x);
  const int bm = (int)fast_div((uint32_t)lid, g.fd_tiles_n);
  const int bn = lid - bm * g.tiles_n;
  const int n0 = bn * BN;
  const int ntile = (g.tiles_m - bm + g.gm - 1) / g.gm;   // >= 1: the grid holds gm <= tiles_m workgroups per channel tile

  const intx4 rs_x = make_rsrc(a.x, (unsigned)((size_t)a.N * a.xs_n * ES));
  const intx4 rs_w = make_rsrc(a.w, (unsigned)((size_t)a.K * a.Kp * ES));
  const size_t out_bytes = (size_t)a.M * a.K * ES;
  const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(a.y, 0, (int)out_bytes, 0x00020000);
  // without a residual operand the descriptor is empty: every load reads zeros, the instruction count stays the same
  const intx4 rs_r = make_rsrc((a.flags & F_RES) ? a.res : a.x, (a.flags & F_RES) ? (unsigned)out_bytes : 0u);

  // ---- this lane's part of every filter slab: LW blocks of 16 rows x 64 B
  const int srow = lane >> 2, sphys = lane & 3;
  unsigned w_off[LW], w_dst[LW];
#pragma unroll
  for (int i = 0; i < LW; ++i) {
    const int fb = wave * LW + i;
    const int plane = fb / (BN / 16), rb = fb % (BN / 16);
    const int row = rb * 16 + srow;
    const int kvl = sphys ^ lds_swizzle(row);
    const int ch = n0 + row;
    const bool mine = fb < FB;   // (uniform) fewer blocks than waves: this wave's filter load is a filler into the dump block
    w_off[i] = (mine && ch < a.K) ? (unsigned)((ch * a.Kp + plane * (BKV * VE) + kvl * VE) * ES) : kOob;
    w_dst[i] = mine ? (unsigned)(plane * WPLANE + rb * 64) * 16u : ~0u;
  }
  // filters of step (cc, t) into ring stage `stage`; live = false: the step does not exist
  auto issue_filter = [&](int i, int cc, int t, int stage, bool live) {
    const unsigned voff = (live && w_off[i] != kOob) ? w_off[i] + (unsigned)((t * a.C + cc * CK) * ES) : kOob;
    lds_dma16(rs_w, w_dst[i] != ~0u ? wring_base + (unsigned)(stage * WSTAGE) * 16u + w_dst[i] : dump_base, voff);
  };

  // ---- this lane's part of a halo: blocks (s * NW + wave), s < XS * HB, of the KP * xblk blocks of a unit
  unsigned x_dst[XS * HB];    // LDS byte offset inside a halo buffer
  unsigned x_add[XS * HB];    // byte offset of this lane's k-vector inside a pixel (chunk 0)
  int x_row[XS * HB];         // halo row of this lane in the block
  unsigned x_live = 0;        // (wave-uniform) bit s: the block exists (else the load is a filler into the dump block)
#pragma unroll
  for (int s = 0; s < XS * HB; ++s) {
    const int b = s * NW + wave;
    const int plane = (int)fast_div((uint32_t)b, g.fd_xblk), blk = b - plane * g.xblk;
    const int row = blk * 16 + srow;
    const int kvl = sphys ^ lds_swizzle(row);
    x_row[s] = row;
    x_add[s] = (unsigned)((plane * (BKV * VE) + kvl * VE) * ES);
    x_dst[s] = (unsigned)((plane * g.xblk + blk) * 64) * 16u;
    if (plane < KP) x_live |= 1u << s;
  }
  // byte offset of the input pixel under flat input position gpos (its channel 0), or kOob for padding
  auto in_pixel = [&](int gpos) -> unsigned {
    const int n = (int)fast_div((uint32_t)gpos, g.fd_f);
    const int rem = gpos - n * g.F;
    const int row = (int)fast_div((uint32_t)rem, g.fd_p);
    const int col = rem - row * g.P;
    return (n < a.N && row >= 1 && col >= 1) ? (unsigned)(((n * a.H + row - 1) * a.W + col - 1) * a.C * ES) : kOob;
  };
  unsigned x_pix[XS * HB];    // per block: this lane's pixel of the tile whose halo is loaded next
  auto decode_tile = [&](int tile_m, bool exists) {
#pragma unroll
    for (int s = 0; s < XS * HB; ++s)
      x_pix[s] = (exists && ((x_live >> s) & 1u)) ? in_pixel(tile_m * BM + x_row[s]) : kOob;
  };
  auto issue_halo = [&](int s, int cc, int buf) {   // block s of chunk cc of the decoded tile into halo buffer buf
    const bool live = (x_live >> s) & 1u;
    const unsigned voff = x_pix[s] != kOob ? x_pix[s] + x_add[s] + (unsigned)(cc * CK * ES) : kOob;
    lds_dma16(rs_x, live ? lds_base + (unsigned)(buf * xbuf_slots) * 16u + x_dst[s] : dump_base, voff);
  };

  // ---- prologue: per-channel constants into registers (their table is written behind the first
  //      loads, which need nothing from them), filters of steps 0 and 1, halo of unit 0
  float cst_mul = 1.f, cst_add = 0.f;
  if (tid < BN) {
    const int c = n0 + tid < a.K ? n0 + tid : a.K - 1;
    if constexpr (IS_I8) {
      cst_mul = __builtin_bit_cast(float, (a.flags & F_BIAS) ? a.qbias[c] : 0);
    } else {
      const float sc = (a.flags & F_BN) ? a.scale[c] : 1.f;
      const float sf = (a.flags & F_BN) ? a.shift[c] : 0.f;
      const float b = (a.flags & F_BIAS) ? a.bias[c] : 0.f;
      cst_mul = sc;
      cst_add = b * sc + sf;   // (acc + b) * sc + sf
    }
  }
#pragma unroll
  for (int i = 0; i < LW; ++i) issue_filter(i, 0, 0, 0, true);
  decode_tile(bm, true);
#pragma unroll
  for (int s = 0; s < XS * HB; ++s) issue_halo(s, 0, 0);
  // the FA - 1 slots in front of step 0 hold L loads like every later one: the filters of steps 1 .. FA - 1
  // (a unit has nine steps and FA <= 7, so they exist) and HB fillers each
#pragma unroll
  for (int f = 1; f < FA; ++f) {
#pragma unroll
    for (int i = 0; i < LW; ++i) issue_filter(i, 0, f, f, true);
#pragma unroll
    for (int h = 0; h < HB; ++h) lds_dma16(rs_x, dump_base, kOob);
  }
  __builtin_amdgcn_sched_barrier(0);
  if (tid < BN) {   // (the first barrier of the loop orders these writes before any read)
    cst[tid] = cst_mul;
    if constexpr (!IS_I8) cst[BN + tid] = cst_add;
  }

  acc_t acc[TN][TM];
#pragma unroll
  for (int tn = 0; tn < TN; ++tn)
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tn][tm][v] = 0;

  const int lrow = lane & 31, lhalf = lane >> 5;
  const int xrow0 = wm * WTM + lrow;   // halo row of this lane's first pixel at tap (0, 0)

  // ---- epilogue of one tile, on the accumulators where they are
  // (the asm loads below write these registers directly: a temporary would be copied before the data is there)
  typedef typename std::conditional<IS_I8, unsigned, uintx2>::type res_t;
  res_t resv[TM][TN][4];
  auto out_offset = [&](int tile_m, int tm) -> unsigned {   // byte offset of channel 0 of this lane's pixel of block row tm, or kOob
    const int o = tile_m * BM + wm * WTM + tm * 32 + lrow;
    const int n = (int)fast_div((uint32_t)o, g.fd_f);
    const int rem = o - n * g.F;
    const int row = (int)fast_div((uint32_t)rem, g.fd_p);
    const int col = rem - row * g.P;
    return (o < g.Mflat && row < a.H && col < a.W) ? (unsigned)(((n * a.H + row) * a.W + col) * a.K * ES) : kOob;
  };
  // issues the R residual loads of a tile (real = false: out-of-range fillers that read zeros)
  auto fetch_residual = [&](int tile_m, bool real) {
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
      const unsigned po = real ? out_offset(tile_m, tm) : kOob;
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int ch = n0 + wn * WTN + tn * 32 + 8 * q4 + 4 * lhalf;
          const unsigned off = (po != kOob && ch < a.K) ? po + (unsigned)(ch * ES) : kOob;
          if constexpr (IS_I8) {
            asm volatile("buffer_load_dword %0, %1, %2, 0 offen" : "=v"(resv[tm][tn][q4]) : "v"(off), "s"(rs_r) : "memory");
          } else {
            asm volatile("buffer_load_dwordx2 %0, %1, %2, 0 offen" : "=v"(resv[tm][tn][q4]) : "v"(off), "s"(rs_r) : "memory");
          }
        }
    }
  };
  // behind the wait that has them landed: from here on the registers hold values the compiler may use
  auto residual_landed = [&]() {
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) asm volatile("" : "+v"(resv[tm][tn][q4]));
  };
  const ClipBounds qb = clip_bounds(a, a.flags & F_RELU);
  auto finish_tile = [&](int tile_m) {
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
      const unsigned po = out_offset(tile_m, tm);
#pragma unroll
      for (int tn = 0; tn < TN; ++tn)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          const int cb = wn * WTN + tn * 32 + 8 * q4 + 4 * lhalf;   // first of the lane's four channels, within the tile
          const int ch = n0 + cb;
          const unsigned off = (po != kOob && ch < a.K) ? po + (unsigned)(ch * ES) : kOob;
          const float4 c0 = *reinterpret_cast<const float4*>(cst + cb);
          if constexpr (IS_I8) {
            const int ib[4] = {__builtin_bit_cast(int, c0.x), __builtin_bit_cast(int, c0.y), __builtin_bit_cast(int, c0.z),
                               __builtin_bit_cast(int, c0.w)};
            const unsigned rv = (unsigned)resv[tm][tn][q4];
            int q[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int t = acc[tn][tm][4 * q4 + e] + ib[e] + (int)(int8_t)(rv >> (8 * e)) * (1 << a.lshift);
              q[e] = shift_round_clip<false>(t, a, qb);   // (the exact form: this kernel runs only where a caller forces it)
            }
            __builtin_amdgcn_raw_buffer_store_b32(pack_low_bytes(q[0], q[1], q[2], q[3]), rs_y, (int)off, 0, 0);
          } else {
            const float4 c1 = *reinterpret_cast<const float4*>(cst + BN + cb);
            const float m4[4] = {c0.x, c0.y, c0.z, c0.w}, a4[4] = {c1.x, c1.y, c1.z, c1.w};
            const half4v rh = __builtin_bit_cast(half4v, (uintx2)resv[tm][tn][q4]);
            half4v hv;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              float t = acc[tn][tm][4 * q4 + e] * m4[e] + a4[e];
              t += (float)rh[e];
              if (a.flags & F_RELU) t = t > 0.f ? t : 0.f;
              hv[e] = (_Float16)t;
            }
            __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(uintx2, hv), rs_y, (int)off, 0, 0);
          }
        }
    }
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[tn][tm][v] = 0;
  };

  // the constants table is LDS traffic of this workgroup only; the first barrier of the loop orders it
  uint4 wfd[DK][TN], xfd[DK][TM];   // operands of the carried k-steps
  bool carried = false;
  int ubuf = 0;                     // halo buffer of the current unit
  int stage = 0;                    // ring stage of the current step's filters
  for (int j = 0; j < ntile; ++j) {
    const int tile_m = bm + j * g.gm;
    for (int cc = 0; cc < g.ncc; ++cc) {
      const bool last_cc = cc + 1 == g.ncc;
      // the unit whose halo is loaded behind this unit's taps: the next chunk of this tile, or chunk 0 of the next tile
      const int ncc_next = last_cc ? 0 : cc + 1;
      const bool next_unit = !last_cc || j + 1 < ntile;
      if (last_cc) decode_tile(tile_m + g.gm, j + 1 < ntile);
      const uint4* xb = lds + ubuf * xbuf_slots;
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        if (t == 9 - FA) {   // the tile's residual operand (fillers unless this is the tile's last unit)
          __builtin_amdgcn_sched_barrier(0);
          fetch_residual(tile_m, last_cc);
          __builtin_amdgcn_sched_barrier(0);
        }
        // How many younger memory instructions may be pending once this step's operands have landed:
        // the FA - 1 slots behind the one that fetched this step's filters, the residual loads while
        // they are younger than that slot (the unit's last FA steps), the previous tile's stores
        // while they are (steps 1 .. FA of a tile that is not the workgroup's first).
        {
          const bool res_in = t >= 9 - FA;                                   // (compile-time once the tap loop is unrolled)
          const bool st_in = t >= 1 && t <= FA && j > 0 && cc == 0;
          if (res_in && st_in) wait_loads<WBASE + 2 * NRES>();
          else if (res_in || st_in) wait_loads<WBASE + NRES>();
          else wait_loads<WBASE>();
        }
        if (t == 0 && j > 0 && cc == 0) residual_landed();   // (this wait is the first that covers them)
        __builtin_amdgcn_s_barrier();
        const uint4* ws = wring + stage * WSTAGE;
        const int xrow = xrow0 + (t / 3) * g.P + (t % 3);   // the tap is a shift of the halo rows
        const int xs = lds_swizzle(xrow);                   // unchanged by the + 32 of the next block
        auto fetch = [&](int k, uint4(&wf)[TN], uint4(&xf)[TM]) {
          const int kq = 2 * (k & 1) + lhalf;
#pragma unroll
          for (int tn = 0; tn < TN; ++tn) wf[tn] = ws[(k >> 1) * WPLANE + lds_slot(wn * WTN + tn * 32 + lrow, kq)];
#pragma unroll
          for (int tm = 0; tm < TM; ++tm) xf[tm] = xb[(k >> 1) * xplane + (xrow + tm * 32) * BKV + (kq ^ xs)];
        };
        // the slot of this step: filters of the step FA ahead (into the stage the previous step has
        // just been read out of), block(s) of the next unit's halo
        const int t2 = (t + FA) % 9;
        const int cc2 = t + FA < 9 ? cc : ncc_next;
        const bool live2 = t + FA < 9 || next_unit;
        const int fill = stage == 0 ? NSW - 1 : stage - 1;
        auto issue_slot = [&](int i) {
          if (i < LW) {
            issue_filter(i, cc2, t2, fill, live2);
          } else {
            const int h = i - LW;
            if (t < XS && next_unit) issue_halo(t * HB + h, ncc_next, ubuf ^ 1);
            else lds_dma16(rs_x, dump_base, kOob);
          }
        };
        uint4 wf[HK][TN], xf[HK][TM];
#pragma unroll
        for (int k = 0; k < HK; ++k) fetch(k, wf[k], xf[k]);
        if (carried) {
#pragma unroll
          for (int k = 0; k < DK; ++k)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
              for (int tm = 0; tm < TM; ++tm) {
                acc[tn][tm] = Mma<IS_I8>::mma(wfd[k][tn], xfd[k][tm], acc[tn][tm]);
                const int i = (k * TN + tn) * TM + tm;
                if (i < L) {
                  __builtin_amdgcn_sched_barrier(0);
                  issue_slot(i);
                  __builtin_amdgcn_sched_barrier(0);
                }
              }
#pragma unroll
          for (int i = DK * TM * TN; i < L; ++i) issue_slot(i);   // (more loads than carried matrix instructions)
        } else {
#pragma unroll
          for (int i = 0; i < L; ++i) issue_slot(i);
        }
        if (j > 0 && cc == 0 && t == 0) {   // (uniform) the previous tile is complete: finish it, start this one from zero
          __builtin_amdgcn_sched_barrier(0);
          finish_tile(tile_m - g.gm);
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int k = 0; k < DK; ++k) fetch(HK + k, wfd[k], xfd[k]);
#pragma unroll
        for (int k = 0; k < HK; ++k)
#pragma unroll
          for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = Mma<IS_I8>::mma(wf[k][tn], xf[k][tm], acc[tn][tm]);
        carried = true;
        stage = stage + 1 == NSW ? 0 : stage + 1;
      }
      ubuf ^= 1;
    }
  }
  // the last tile's carried products, then its epilogue
  wait_loads<0>();   // its residual operand (and the trailing out-of-range loads, which still write zeros into LDS)
  residual_landed();
#pragma unroll
  for (int k = 0; k < DK; ++k)
#pragma unroll
    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
      for (int tm = 0; tm < TM; ++tm) acc[tn][tm] = Mma<IS_I8>::mma(wfd[k][tn], xfd[k][tm], acc[tn][tm]);
  finish_tile(bm + (ntile - 1) * g.gm);
}

struct StreamTile {
  int waves_m, waves_n, tm, tn, hb, wgs, fa;
  constexpr int bm() const { return waves_m * tm * 32; }
  constexpr int bn() const { return waves_n * tn * 32; }
  constexpr int nw() const { return waves_m * waves_n; }
};
// 256 x 64 with eight waves, one workgroup per compute unit; 128 x 64 with four waves, two per compute unit
// and the eight-wave tile with filters fetched five steps ahead (a six-stage ring)
constexpr StreamTile kStream[] = {{4, 2, 2, 1, 1, 1, 2}, {2, 2, 2, 1, 2, 2, 2}, {4, 2, 2, 1, 2, 1, 5}};
constexpr int kNumStream = 3;
constexpr int kCUs = 256;

int stream_planes(const ConvArgs& a, bool is_i8) {
  const int ve = is_i8 ? 16 : 8;
  return a.C % (2 * BKV * ve) == 0 ? 2 : 1;
}

bool stream_geom(const ConvArgs& a, bool is_i8, int v, StreamGeom& g, size_t& lds_bytes, int& grid) {
  const StreamTile& t = kStream[v];
  const int kp = stream_planes(a, is_i8), ve = is_i8 ? 16 : 8;
  g.P = a.W + 1;
  g.F = (a.H + 1) * g.P;
  if ((long)a.N * g.F + t.bm() + 2 * g.P + 2 > 0x3fffffffL) return false;
  g.Mflat = a.N * g.F;
  const int rows = t.bm() + 2 * g.P + 2;
  g.xblk = (rows + 15) / 16;
  g.ncc = a.C / (kp * BKV * ve);
  if (kp * g.xblk > halo_slots(t.fa) * t.hb * t.nw()) return false;   // a halo must fit its load slots
  g.tiles_m = (g.Mflat + t.bm() - 1) / t.bm();
  g.tiles_n = (a.K + t.bn() - 1) / t.bn();
  const int slots = a.max_wgs > 0 ? a.max_wgs : kCUs * t.wgs;
  g.gm = slots / g.tiles_n;
  if (g.gm < 1) g.gm = 1;
  if (g.gm > g.tiles_m) g.gm = g.tiles_m;
  grid = g.gm * g.tiles_n;
  g.fd_f = make_fastdiv((uint32_t)g.F);
  g.fd_p = make_fastdiv((uint32_t)g.P);
  g.fd_xblk = make_fastdiv((uint32_t)g.xblk);
  g.fd_tiles_n = make_fastdiv((uint32_t)g.tiles_n);
  const size_t slots16 = (size_t)2 * kp * g.xblk * 64 + (size_t)ring_stages(t.fa) * kp * t.bn() * BKV + 64 + (size_t)t.bn() / 2;
  lds_bytes = slots16 * 16;
  return lds_bytes <= (size_t)(160 * 1024) / t.wgs;
}

template <bool IS_I8, int WM, int WN, int TM, int TN, int KP, int HB, int WGS, int FA>
hipError_t launch_stream_one(const ConvArgs& a, const StreamGeom& g, size_t lds_bytes, int grid, hipStream_t st) {
  auto kern = conv3x3_stream_kernel<IS_I8, WM, WN, TM, TN, KP, HB, WGS, FA>;
  static std::atomic<bool> raised{false};  // dynamic LDS above the default limit has to be asked for once per kernel
  if (!raised.load(std::memory_order_acquire)) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                             160 * 1024);
    if (e != hipSuccess) return e;
    raised.store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * WM * WN), lds_bytes, st, a, g);
  return hipGetLastError();
}

template <bool IS_I8>
hipError_t launch_stream_typed(const ConvArgs& a, const StreamGeom& g, size_t lds_bytes, int grid, int v, int kp, hipStream_t st) {
  switch (v) {
    case 0: return kp == 2 ? launch_stream_one<IS_I8, 4, 2, 2, 1, 2, 1, 1, 2>(a, g, lds_bytes, grid, st)
                           : launch_stream_one<IS_I8, 4, 2, 2, 1, 1, 1, 1, 2>(a, g, lds_bytes, grid, st);
    case 1: return kp == 2 ? launch_stream_one<IS_I8, 2, 2, 2, 1, 2, 2, 2, 2>(a, g, lds_bytes, grid, st)
                           : launch_stream_one<IS_I8, 2, 2, 2, 1, 1, 2, 2, 2>(a, g, lds_bytes, grid, st);
    default: return kp == 2 ? launch_stream_one<IS_I8, 4, 2, 2, 1, 2, 2, 1, 5>(a, g, lds_bytes, grid, st)
                            : launch_stream_one<IS_I8, 4, 2, 2, 1, 1, 2, 1, 5>(a, g, lds_bytes, grid, st);
  }
}

}  // namespace

int conv_stream_variant_count() { return kNumStream; }

// 3x3, stride 1, pad 1, plain NHWC in and out, whole chunks of channels, K % 8 == 0, deterministic rounding.
bool conv_stream_supported(const ConvArgs& a, bool is_i8, int v) {
  if (v < 0 || v >= kNumStream) return false;
  const int es = is_i8 ? 1 : 2, ve = is_i8 ? 16 : 8;
  if (a.R != 3 || a.S != 3 || a.sh != 1 || a.sw != 1 || a.ph != 1 || a.pw != 1) return false;
  if (a.xs_w != a.C || a.xs_h != a.W * a.C || a.xs_n != a.H * a.W * a.C) return false;
  if (a.C % (BKV * ve) != 0 || (a.K & 7) != 0 || a.round_mode == ROUND_STOCHASTIC || a.nseg || a.split > 1 || a.pool) return false;
  if (a.qmode != QMODE_SHIFT) return false;   // the other scaling rules of the quantized tail live in the one-tile kernels
  if ((size_t)a.N * a.xs_n * es > 0x7fffffffu || (size_t)a.K * a.Kp * es > 0x7fffffffu || (size_t)a.M * a.K * es > 0x7fffffffu)
    return false;
  StreamGeom g;
  size_t lds_bytes;
  int grid;
  return stream_geom(a, is_i8, v, g, lds_bytes, grid);
}

// The variant the heuristic takes, or -1 to leave the layer to the other kernels.  Measured on the
// ResNet-18 layers (fp16 batch 32 / int8 batch 16) every variant is slower than the one-tile-per-
// workgroup kernels (64 channels at 56 x 56: 21.3 / 18.2 / 23.1 us against 16.7; 128 at 28 x 28: 15.8 /
// 17.6 / 17.2 against 12.4 - 15.7; int8 9.5 against 7.5): a step of the eight-wave tile reads 96 KB of
// operands out of LDS, 750 clocks at the 128 B/clk the LDS delivers, against 512 clocks of matrix
// work, and the 8-byte stores of the in-place epilogue cost a quarter of the run.  So no layer is
// given to this kernel unless a caller forces it (relay_set_conv_tile(200 + variant)).
int conv_stream_pick(const ConvArgs& a, bool is_i8) {
  (void)a;
  (void)is_i8;
  return -1;
}

void conv_stream_kernel_name(const ConvArgs& a, bool is_i8, int v, char* buf, size_t len) {
  const StreamTile& t = kStream[v];
  snprintf(buf, len, "conv3x3_stream_kernel<%s, %d, %d, %d, %d, %d, %d, %d, %d>", is_i8 ? "true" : "false", t.waves_m, t.waves_n,
           t.tm, t.tn, stream_planes(a, is_i8), t.hb, t.wgs, t.fa);
}

hipError_t launch_conv_stream(const ConvArgs& a, bool is_i8, int v, hipStream_t st) {
  StreamGeom g;
  size_t lds_bytes;
  int grid;
  if (!stream_geom(a, is_i8, v, g, lds_bytes, grid)) return hipErrorInvalidValue;
  const int kp = stream_planes(a, is_i8);
  return is_i8 ? launch_stream_typed<true>(a, g, lds_bytes, grid, v, kp, st)
               : launch_stream_typed<false>(a, g, lds_bytes, grid, v, kp, st);
}

}  // namespace relay
