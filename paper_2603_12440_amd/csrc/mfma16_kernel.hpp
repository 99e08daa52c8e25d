// Matrix-core GEMM for gfx950 on the 16x16x32 MFMA shape: 16-bit operands (bf16 / fp16),
// fp32 accumulate.
//
//   C = act(A . B + bias),  A row-major (K contiguous), B column-major (K contiguous: the
//   "weight" matrix stored N x K), C row-major.
//
// Same data path as mfma_kernel.hpp (direct-to-LDS slabs of 64 columns of K, two stages,
// XOR-swizzled 16-byte chunks, 16-byte fragment reads, accumulators in AccVGPRs, hand-placed
// waits), but the products are issued as v_mfma_f32_16x16x32: measured on an MI355X, whose
// matrix pipes are power-limited, that shape delivers about a tenth more FLOP/s than
// v_mfma_f32_32x32x16 at the same power (it reads and writes a quarter of the accumulator
// registers per instruction and sums 32 products before touching them).  What else differs:
//   * a k-step is 32 columns of K and is multiplied in G sub-steps of MT/G row fragments
//     times all NT column fragments, so that the fragment registers are double-buffered per
//     sub-step (A) and per k-step (B) instead of per whole k-step of both;
//   * the global -> LDS loads of a slab are spread over the sub-steps that follow the
//     hand-over instead of being issued in one burst;
//   * with two waves per SIMD, each wave lowers its priority as it advances from one
//     hand-over to the next, so that the wave that is behind gets the matrix pipe and the
//     two alternate sub-step by sub-step instead of one running ahead to the barrier.
// Paper taxonomy (Sec. 3.2): d_mem = 3, d_algo = 1 (fused post-op), d_sync = 1.
#pragma once

#include <type_traits>

#include "mfma_kernel.hpp"

namespace mi355gemm {

template <typename T> struct Frag16;
template <> struct Frag16<bf16_t> {
  static __device__ __forceinline__ void mfma(const u32x4_t& x, const u32x4_t& y, f32x4_t& c) {
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(x), "v"(y));
  }
};
template <> struct Frag16<f16_t> {
  static __device__ __forceinline__ void mfma(const u32x4_t& x, const u32x4_t& y, f32x4_t& c) {
    asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(c) : "v"(x), "v"(y));
  }
};

// Chunk c (16 bytes) of slab row r is stored at chunk slot c ^ swz16(r).  A fragment read
// touches 16 consecutive rows at one logical chunk per quarter wave; rows are 128 bytes
// apart (32 banks), so row parity picks the half of the banks and (r >> 1) & 7 the 16-byte
// slot within it: the 16 rows cover all 64 banks once.  The key uses row bits 1..3 only, so
// fragments 16 rows apart differ by a constant offset.
__device__ __forceinline__ int swz16(int r) { return (r >> 1) & 7; }

// ---- the instruction order of one sub-step, generated at compile time ---------------------
// A sub-step multiplies MA row fragments with NT column fragments.  While it runs, the reads
// for the next sub-step are requested, one behind each of its first MFMAs: MA row fragments
// and, when the next sub-step begins a new k-step, the NT column fragments too (WITH_B).
// Its own MFMAs run in the order in which their operands were requested one sub-step earlier.
template <int MA, int NT, bool WITH_B>
struct SubOrder {
  static constexpr int kReads = MA + (WITH_B ? NT : 0), kMfma = MA * NT;
  struct Tables {
    int r_isb[kReads], r_idx[kReads];
    int mm[kMfma], nn[kMfma];
    int need[kMfma];        // request position of the later of MFMA i's operands (-1: resident)
  };
  static constexpr Tables make() {
    Tables t{};
    int pos_a[MA] = {}, pos_b[NT] = {};
    for (int n = 0; n < NT; ++n) pos_b[n] = -1;
    int c = 0;
    if (WITH_B) {
      // a0 b0 b1 a1 b2 a2 ...: the first MFMAs can start after two reads
      for (int i = 0; i < (MA > NT ? MA : NT); ++i) {
        if (i == 0) {
          t.r_isb[c] = 0; t.r_idx[c] = 0; pos_a[0] = c++;
          t.r_isb[c] = 1; t.r_idx[c] = 0; pos_b[0] = c++;
        } else {
          if (i < NT) { t.r_isb[c] = 1; t.r_idx[c] = i; pos_b[i] = c++; }
          if (i < MA) { t.r_isb[c] = 0; t.r_idx[c] = i; pos_a[i] = c++; }
        }
      }
    } else {
      for (int i = 0; i < MA; ++i) { t.r_isb[c] = 0; t.r_idx[c] = i; pos_a[i] = c++; }
    }
    bool used[kMfma] = {};
    for (int i = 0; i < kMfma; ++i) {
      int best = -1, best_key = 0;
      for (int q = 0; q < kMfma; ++q) {
        if (used[q]) continue;
        const int m = q / NT, n = q % NT;
        const int p = pos_a[m] > pos_b[n] ? pos_a[m] : pos_b[n];
        const int key = (p + 1) * kMfma + q;
        if (best < 0 || key < best_key) { best = q; best_key = key; }
      }
      used[best] = true;
      t.mm[i] = best / NT;
      t.nn[i] = best % NT;
      t.need[i] = best_key / kMfma - 1;
    }
    return t;
  }
  static constexpr Tables t = make();
};

template <typename T, int BM, int BN, int WM, int WN, int G>
struct Mfma16Tile {
  static constexpr int BK = 64, NSTAGE = 2;
  static constexpr int kWaves = WM * WN, kThreads = 64 * kWaves;
  static constexpr int WTM = BM / WM, WTN = BN / WN;     // per-wave block
  static constexpr int MT = WTM / 16, NT = WTN / 16;     // 16x16 MFMA tiles per wave
  static constexpr int MA = MT / G;                      // row fragments per sub-step
  static constexpr int KK = BK / 32;                     // k-steps (32 columns) per slab
  static constexpr int NSUB = KK * G;                    // sub-steps per slab
  static constexpr int ROWB = BK * 2;                    // bytes per slab row
  static constexpr int CPR = ROWB / 16, RPI = 64 / CPR;  // chunks per row, rows per wave-wide load
  static constexpr int A_LOADS = BM / RPI / kWaves, B_LOADS = BN / RPI / kWaves;
  static constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
  // the epilogue's staging area of a persistent workgroup: one 16-row band of every wave's block in fp32
  static constexpr int EPI_BYTES = kWaves * 16 * WTN * 4;
  static_assert(sizeof(T) == 2, "16-bit operands");
  static_assert(BM % (RPI * kWaves) == 0 && BN % (RPI * kWaves) == 0, "slab rows must divide over waves");
  static_assert(WTM % 16 == 0 && WTN % 16 == 0 && MT % G == 0, "wave block in whole sub-steps");
  static_assert(NSUB % 2 == 0, "the row-fragment double buffer alternates per sub-step");
  static_assert(MA * NT >= MA + NT, "a sub-step issues one fragment read behind each MFMA");
  static_assert(LDS_BYTES + EPI_BYTES <= 160 * 1024, "LDS budget");
};

// T: operand type; TO: the 16-bit output type (outputs may also be fp32: MfmaArgs::c_f32).
// PERSIST: a workgroup walks over several tiles (tile ids blockIdx.x, blockIdx.x + gridDim.x,
// ...) as one software pipeline: the slabs of the next tile are requested while the last slabs
// of the current one are multiplied, and land while its epilogue runs, which stages C through an
// LDS region of its own.  Needs K to be a whole number of slabs, at least two.
template <typename T, typename TO, int BM, int BN, int WM, int WN, int G, bool PERSIST>
__global__ __launch_bounds__(64 * WM * WN) void mfma16_gemm_kernel(MfmaArgs p) {
  typedef Mfma16Tile<T, BM, BN, WM, WN, G> Cfg;
  constexpr int MT = Cfg::MT, NT = Cfg::NT, MA = Cfg::MA, CPR = Cfg::CPR, RPI = Cfg::RPI;
  constexpr int ROWB = Cfg::ROWB, BK = Cfg::BK, KK = Cfg::KK, NSUB = Cfg::NSUB;
  constexpr bool kTwoPerSimd = Cfg::kWaves > 4;          // two waves share a SIMD: alternate by priority

  __shared__ __attribute__((aligned(1024))) unsigned char smem[Cfg::LDS_BYTES + (PERSIST ? Cfg::EPI_BYTES : 0)];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  // One tile per workgroup: the batch is the grid's second index.  A persistent workgroup walks over
  // the tiles of every problem of the batch (tile id = problem * n_tiles + tile within the problem);
  // `batch` is then the problem of the tile being written out.
  int batch = PERSIST ? 0 : (int)blockIdx.y;
  const int n_tiles = p.tiles_m * p.tiles_n;
  const int total_tiles = PERSIST ? n_tiles * p.batches : n_tiles;
  // A batch on persistent workgroups (xcd_remap == 2; grid and tile count multiples of 8): the 8 XCDs
  // (round-robin dispatch: XCD = tile id mod 8) each take a contiguous run of the problems, so that the
  // tiles of one problem, which share its panels, meet in one L2 instead of fetching them 8 times.
  auto logical_tile = [&](int vid) __attribute__((always_inline)) {
    return p.xcd_remap == 2 ? (vid & 7) * (total_tiles >> 3) + (vid >> 3) : vid;
  };

  // ---- global -> LDS addressing (as in mfma_kernel.hpp, with this kernel's swizzle) -------
  // Load q of this wave fills LDS bytes [slab + (wave*LOADS + q)*1024, +1024): lane l writes
  // 16 bytes at +16*l, i.e. slab row (wave*LOADS+q)*RPI + l/CPR, slot l%CPR, which must
  // receive logical chunk slot ^ swz16(row).  Rows past the matrix edge are clamped to the
  // last valid row (their results are never stored).
  // The tile the loads work on (it runs ahead of the tile being multiplied):
  const char* ld_a;                              // first byte of the next slab to request, A and B
  const char* ld_b;
  uint32_t a_off[Cfg::A_LOADS], b_off[Cfg::B_LOADS];
  // (`ln`: the lane id; a persistent workgroup recomputes the offsets from a fresh copy of it after
  // each epilogue, so that they need not stay in registers across it.)  Leaves ld_a / ld_b at slab `kt`.
  auto load_tile = [&](int vid, int ln, int kt) __attribute__((always_inline)) {
    int tm, tn;
    const int lid = PERSIST ? logical_tile(vid) : vid;
    const int lb = PERSIST ? lid / n_tiles : batch;          // the problem this tile belongs to
    tile_coords(p, PERSIST ? lid - lb * n_tiles : vid, n_tiles, tm, tn);
    const int r0 = tm * BM, c0 = tn * BN;
    ld_a = (const char*)((const T*)p.A + (int64_t)lb * p.stride_a + (int64_t)r0 * p.lda) + (int64_t)kt * ROWB;
    ld_b = (const char*)((const T*)p.B + (int64_t)lb * p.stride_b + (int64_t)c0 * p.ldb) + (int64_t)kt * ROWB;
#pragma unroll
    for (int q = 0; q < Cfg::A_LOADS; ++q) {
      const int r = (wave * Cfg::A_LOADS + q) * RPI + ln / CPR;
      const int c = (ln % CPR) ^ swz16(r);
      const int rr = min(r, p.M - 1 - r0);
      a_off[q] = (uint32_t)(((int64_t)rr * p.lda + c * 8) * 2);
    }
#pragma unroll
    for (int q = 0; q < Cfg::B_LOADS; ++q) {
      const int r = (wave * Cfg::B_LOADS + q) * RPI + ln / CPR;
      const int c = (ln % CPR) ^ swz16(r);
      const int rr = min(r, p.N - 1 - c0);
      b_off[q] = (uint32_t)(((int64_t)rr * p.ldb + c * 8) * 2);
    }
  };
  load_tile(blockIdx.x, lane, 0);
  const char* const Ab = ld_a;                   // (the first tile's panels: the one-tile path indexes them by slab)
  const char* const Bb = ld_b;

  const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_uchar_t*)smem;
  constexpr int kLoads = Cfg::A_LOADS + Cfg::B_LOADS;
  // Where the loads of one slab go and come from: the slab's first byte in A and in B and the
  // LDS addresses of this wave's share of the stage's A and B parts.  All four are wave-uniform
  // and are read back through the scalar unit once per slab, far from the loads that use them.
  struct SlabIo { const char* ga; const char* gb; uint32_t la, lb; };
  auto uniform_ptr = [](const char* q) __attribute__((always_inline)) {
    const uint64_t gv = (uint64_t)q;
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(gv >> 32));
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)gv);
    return (const char*)(((uint64_t)hi << 32) | (uint64_t)lo);
  };
  auto slab_io_at = [&](const char* ga, const char* gb, int st) __attribute__((always_inline)) {
    SlabIo io;
    io.ga = uniform_ptr(ga);
    io.gb = uniform_ptr(gb);
    io.la = (uint32_t)__builtin_amdgcn_readfirstlane((int)(lds_base + st * Cfg::STAGE_BYTES + wave * (Cfg::A_LOADS * 1024)));
    io.lb = (uint32_t)__builtin_amdgcn_readfirstlane(
        (int)(lds_base + st * Cfg::STAGE_BYTES + Cfg::A_BYTES + wave * (Cfg::B_LOADS * 1024)));
    return io;
  };
  auto slab_io = [&](int kt, int st) __attribute__((always_inline)) {
    return slab_io_at(Ab + (int64_t)kt * ROWB, Bb + (int64_t)kt * ROWB, st);
  };
  // One direct-to-LDS load (scalar base + 32-bit lane offset; M0 = LDS destination of the wave,
  // lane l lands at M0 + 16*l): q < A_LOADS fills the A slab, the rest the B slab.  M0 is written
  // by a scalar add; one wait state must pass before the load reads it.  The address pair must
  // not have been written by a vector instruction within five cycles of the load (the hardware
  // does not check): slab_io produces it long before, and the build scans the generated code for it.
  auto issue_one_load = [&](int q, const SlabIo& io) __attribute__((always_inline)) {
    if (q < Cfg::A_LOADS) {
      asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3"
                   :: "s"(io.la), "n"(q * 1024), "v"(a_off[q < Cfg::A_LOADS ? q : 0]), "s"(io.ga) : "memory", "m0", "scc");
    } else {
      asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3"
                   :: "s"(io.lb), "n"((q - Cfg::A_LOADS) * 1024), "v"(b_off[q >= Cfg::A_LOADS ? q - Cfg::A_LOADS : 0]), "s"(io.gb) : "memory", "m0", "scc");
    }
  };

  // K tail: chunks past K must read as zero, which a direct-to-LDS load cannot do, so that one
  // slab goes through registers.  (K is a multiple of 8: chunks are never split.)
  auto issue_loads_tail = [&](int kt, int stage) __attribute__((always_inline)) {
    const int kvalid = p.K - kt * BK;
    const char* ga = Ab + (int64_t)kt * ROWB;
    const char* gb = Bb + (int64_t)kt * ROWB;
    unsigned char* sa = smem + stage * Cfg::STAGE_BYTES + wave * (Cfg::A_LOADS * 1024);
    unsigned char* sb = smem + stage * Cfg::STAGE_BYTES + Cfg::A_BYTES + wave * (Cfg::B_LOADS * 1024);
#pragma unroll
    for (int q = 0; q < Cfg::A_LOADS; ++q) {
      const int r = (wave * Cfg::A_LOADS + q) * RPI + lane / CPR;
      const int c = (lane % CPR) ^ swz16(r);
      u32x4_t v = {0u, 0u, 0u, 0u};
      if (c * 8 < kvalid) v = *(const u32x4_t*)(ga + a_off[q]);
      *(u32x4_t*)(sa + q * 1024 + lane * 16) = v;
    }
#pragma unroll
    for (int q = 0; q < Cfg::B_LOADS; ++q) {
      const int r = (wave * Cfg::B_LOADS + q) * RPI + lane / CPR;
      const int c = (lane % CPR) ^ swz16(r);
      u32x4_t v = {0u, 0u, 0u, 0u};
      if (c * 8 < kvalid) v = *(const u32x4_t*)(gb + b_off[q]);
      *(u32x4_t*)(sb + q * 1024 + lane * 16) = v;
    }
  };

  // ---- LDS -> fragment addressing ---------------------------------------------------------
  // MFMA 16x16x32 operand: lane l holds 8 consecutive k of row (l % 16), k-octet l / 16 of the
  // step's four.  Fragment m of the wave is 16*m rows further on: a constant offset.  The
  // address registers point into the stage being read and move to the other stage at each
  // hand-over (one vector add each), so a fragment read needs no address arithmetic.
  uint32_t a_rd[KK], b_rd[KK];
  int rd_delta;                                  // to the other stage (alternates in sign)
  // point the address registers into stage `st` (`ln`: the lane id, see load_tile)
  auto set_read_stage = [&](int st, int ln) __attribute__((always_inline)) {
    const int fr = ln & 15, fo = ln >> 4;
    const int a_row = wm * Cfg::WTM + fr;
    const int b_row = wn * Cfg::WTN + fr;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const int c = kk * 4 + fo;
      a_rd[kk] = lds_base + st * Cfg::STAGE_BYTES + a_row * ROWB + ((c ^ swz16(a_row)) * 16);
      b_rd[kk] = lds_base + st * Cfg::STAGE_BYTES + Cfg::A_BYTES + b_row * ROWB + ((c ^ swz16(b_row)) * 16);
    }
    rd_delta = st ? -Cfg::STAGE_BYTES : Cfg::STAGE_BYTES;
  };
  set_read_stage(0, lane);
  auto flip_read_stage = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) { a_rd[kk] += rd_delta; b_rd[kk] += rd_delta; }
    rd_delta = -rd_delta;
  };

  f32x4_t acc[MT][NT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[m][n][r] = 0.0f;

  // Fragment registers: row fragments double-buffered per sub-step, column fragments per k-step.
  u32x4_t af[2][MA], bf[2][NT];

  // Sub-step u of a slab: k-step u / G, row group u % G.
  // the i-th read of the requests made for sub-step `u` (from the stage the address registers point into)
  auto read_one = [&](auto u_c, int i) __attribute__((always_inline)) {
    constexpr int u = decltype(u_c)::value;
    constexpr int kk = u / G, g = u % G;
    typedef SubOrder<MA, NT, g == 0> Ord;
    const int idx = Ord::t.r_idx[i];
    if (Ord::t.r_isb[i]) lds_read_b128(bf[kk & 1][idx], b_rd[kk], idx * (16 * ROWB));
    else lds_read_b128(af[u & 1][idx], a_rd[kk], (g * MA + idx) * (16 * ROWB));
  };
  auto read_all = [&](auto u_c) __attribute__((always_inline)) {
    constexpr int u = decltype(u_c)::value;
    typedef SubOrder<MA, NT, (u % G) == 0> Ord;
#pragma unroll
    for (int i = 0; i < Ord::kReads; ++i) read_one(u_c, i);
  };

  // One sub-step `u`: its MFMAs in the order their operands were requested, preceded by the
  // wait they need (LDS reads return in order; a wait is only issued when an MFMA needs a later
  // request than every MFMA before it); with `reads`, the requests for the next sub-step go out
  // one behind each of the first MFMAs; loads q0 .. q1-1 of the slab `io` are spaced evenly
  // over the MFMAs.
  auto sub_step = [&](auto u_c, bool reads, int q0, int q1, const SlabIo& io, bool do_loads = true) __attribute__((always_inline)) {
    constexpr int u = decltype(u_c)::value;
    constexpr int kk = u / G, g = u % G;
    constexpr int un = (u + 1) % NSUB;                    // the sub-step the reads are for
    typedef SubOrder<MA, NT, g == 0> Ord;                 // how this sub-step's operands were requested
    typedef SubOrder<MA, NT, (un % G) == 0> OrdN;         // this sub-step's own requests
    const int nq = q1 - q0;
    int waited = -1;
#pragma unroll
    for (int i = 0; i < Ord::kMfma; ++i) {
      const int m = Ord::t.mm[i], n = Ord::t.nn[i];
      if (Ord::t.need[i] > waited) {
        // since the needed request: the rest of that sub-step's requests and min(i, kReads) of ours
        const int after = (Ord::kReads - 1 - Ord::t.need[i]) + (reads ? (i < OrdN::kReads ? i : OrdN::kReads) : 0);
        wait_lgkmcnt_dyn(after);                 // (the counter holds 15 at most: larger values wait for 15)
        waited = Ord::t.need[i];
      }
      Frag16<T>::mfma(bf[kk & 1][n], af[u & 1][m], acc[g * MA + m][n]);
      if (reads && i < OrdN::kReads) read_one(std::integral_constant<int, un>(), i);
#pragma unroll
      for (int j = 0; j < nq; ++j)
        if ((int)((j + 0.5f) * Ord::kMfma / nq) == i) {
          if (do_loads) issue_one_load(q0 + j, io);      // (a wave-uniform branch around one statement)
        }
    }
  };
  auto set_prio = [&](int pr) __attribute__((always_inline)) {
    if (!kTwoPerSimd) return;
    switch (pr) {
      case 0: __builtin_amdgcn_s_setprio(0); break;
      case 1: __builtin_amdgcn_s_setprio(1); break;
      case 2: __builtin_amdgcn_s_setprio(2); break;
      default: __builtin_amdgcn_s_setprio(3); break;
    }
  };

  // ---- epilogue of the tile at (row0, col0) ---------------------------------------------------
  auto epilogue = [&](int row0, int col0) __attribute__((always_inline)) {
    // What the epilogue needs of the arguments.  A persistent workgroup reads them from the argument
    // block again for every tile (the kernel's only argument sits at the start of the kernarg segment),
    // so that they do not occupy scalar registers during the K loops.
    typedef __attribute__((address_space(4))) const volatile MfmaArgs kernarg_t;
    MfmaArgs pe = p;
    if constexpr (PERSIST) {
      kernarg_t* pv = (kernarg_t*)__builtin_amdgcn_kernarg_segment_ptr();
      pe.C = pv->C; pe.bias = pv->bias; pe.M = pv->M; pe.N = pv->N; pe.ldc = pv->ldc; pe.stride_c = pv->stride_c;
      pe.stride_bias = pv->stride_bias; pe.has_bias = pv->has_bias; pe.act = pv->act; pe.c_f32 = pv->c_f32;
      pe.c_cached = pv->c_cached; pe.scale = pv->scale;
    }
    // The MFMAs were issued through inline assembly: the compiler inserts none of the wait states
    // a vector-ALU read of a just-written MFMA result needs.  Wait once, and route every
    // accumulator through an (empty) volatile statement placed after the wait.
    asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
      for (int n = 0; n < NT; ++n) asm volatile("" : "+a"(acc[m][n]));

    // ---- epilogue ---------------------------------------------------------------------------
    // Lane l of a 16x16 accumulator tile holds row (l % 16) and, in its four registers, columns
    // 4*(l / 16) .. +3 (the operands go in swapped, column fragment first).  For whole-line
    // stores each wave passes one 16-row band of its block at a time through its own piece of
    // the (now idle) LDS: 8- or 16-byte writes in accumulator order, 16-byte reads in row order.
    const float* bias = pe.has_bias ? pe.bias + (int64_t)batch * pe.stride_bias : nullptr;
    const int act = pe.act;
    auto fresh_lane = []() __attribute__((always_inline)) {
      unsigned z = 0;
      asm volatile("" : "+v"(z));
      return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, z));
    };
    const int elane = fresh_lane();
    const int er = elane & 15, eq = elane >> 4;

    // bias of the 4 columns j .. j+3 (zero past N; j is a multiple of 4); 16-byte loads only when the
    // bias vector of this batch starts at a 16-byte aligned address (the same for every lane)
    const bool bias_vec = (((uintptr_t)bias) & 15) == 0;
    auto bias4 = [&](int j, float (&bv)[4]) __attribute__((always_inline)) {
#pragma unroll
      for (int e = 0; e < 4; ++e) bv[e] = 0.0f;
      if (!bias) return;
      if (j + 3 < pe.N && bias_vec) {
        const f32x4_t b4 = *(const f32x4_t*)(bias + j);
#pragma unroll
        for (int e = 0; e < 4; ++e) bv[e] = b4[e];
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (j + e < pe.N) bv[e] = bias[j + e];
      }
    };

    const bool through_lds = !pe.c_f32 && (pe.ldc % 8 == 0) && (pe.stride_c % 8 == 0) &&
                             (((uintptr_t)pe.C & 15) == 0);
    const bool through_lds32 = pe.c_f32 && (pe.ldc % 4 == 0) && (pe.stride_c % 4 == 0) && (((uintptr_t)pe.C & 15) == 0);
    constexpr int OROWB = Cfg::WTN * 2;           // bytes per 16-bit row of the wave's block (128 or 256)
    constexpr int CH = OROWB / 16;
    constexpr int OROWB32 = Cfg::WTN * 4;         // bytes per fp32 row (256 or 512)
    constexpr int CH32 = OROWB32 / 16;
    constexpr int kShare = Cfg::LDS_BYTES / Cfg::kWaves;
    static_assert(16 * OROWB32 <= kShare, "one 16-row band of the wave block in fp32 must fit the wave's share of LDS");
    static_assert(OROWB == 128 || OROWB == 256, "staging rows of 128 or 256 bytes");
    static_assert(2 * 16 * OROWB <= (PERSIST ? Cfg::EPI_BYTES / Cfg::kWaves : kShare), "two 16-bit bands per wave");
    // staging: this wave's share of the idle slab stages, or of the separate area of a persistent workgroup
    unsigned char* wt = PERSIST ? smem + Cfg::LDS_BYTES + wave * (Cfg::EPI_BYTES / Cfg::kWaves) : smem + wave * kShare;
    // chunk-slot key of staging row r: 128-byte rows alternate between the two halves of the banks,
    // longer rows all start at bank 0
    auto osw = [](int r) __attribute__((always_inline)) { return OROWB == 128 ? ((r >> 1) & 7) : (r & 15); };

    // 16-bit through LDS, pipelined over the 16-row bands of the wave block with two staging
    // buffers: while the rows of band m-1 come back from LDS, the values of band m+1 are computed;
    // a band's stores are on their way to memory while the next one is drained.
    constexpr int kBand16 = 16 * OROWB;             // bytes of one staged band
    constexpr int kIt16 = 16 * CH / 64;             // wave-wide 16-byte accesses per band
    auto drain16_all = [&](auto actf) __attribute__((always_inline)) {
      TO* Cb = (TO*)pe.C + (int64_t)batch * pe.stride_c;
      const int slane = fresh_lane();
      u32x2_t w[NT];
      u32x4_t val[kIt16];
      float bvs[NT][4];                           // the bias of this lane's columns, the same for every band
#pragma unroll
      for (int n = 0; n < NT; ++n) bias4(col0 + wn * Cfg::WTN + n * 16 + eq * 4, bvs[n]);
      auto values = [&](auto m_c) __attribute__((always_inline)) {
        constexpr int m = decltype(m_c)::value;
#pragma unroll
        for (int n = 0; n < NT; ++n) {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = actf(acc[m][n][e] + bvs[n][e]);
          w[n] = u32x2_t{pack2<TO>(v[0], v[1]), pack2<TO>(v[2], v[3])};
        }
      };
      auto write = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < NT; ++n) {
          const int q = n * 2 + (eq >> 1);
          *(u32x2_t*)(wt + buf * kBand16 + er * OROWB + ((q ^ osw(er)) * 16) + (eq & 1) * 8) = w[n];
        }
      };
      auto read = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < kIt16; ++it) {
          const int e = it * 64 + slane;
          const int r = e / CH, q = e % CH;
          val[it] = *(const u32x4_t*)(wt + buf * kBand16 + r * OROWB + ((q ^ osw(r)) * 16));
        }
      };
      // A tile that lies wholly inside C (the common case) stores without per-element tests, from a
      // wave-uniform base with 32-bit lane offsets: the epilogue is bound by instruction issue (two
      // waves per SIMD drain 128 accumulators each), so every address and mask instruction counts.
      const bool inside = row0 + BM <= pe.M && col0 + BN <= pe.N && (int64_t)BM * pe.ldc * 2 < ((int64_t)1 << 31);
      char* const wave_c = (char*)(Cb + (int64_t)(row0 + wm * Cfg::WTM) * pe.ldc + col0 + wn * Cfg::WTN);
      const uint32_t band_step = (uint32_t)(16 * pe.ldc * 2);
      uint32_t lane_off[kIt16];
#pragma unroll
      for (int it = 0; it < kIt16; ++it) {
        const int e = it * 64 + slane;
        lane_off[it] = (uint32_t)((e / CH) * (int)pe.ldc * 2 + (e % CH) * 16);
      }
      auto store = [&](int m) __attribute__((always_inline)) {
        if (inside) {
#pragma unroll
          for (int it = 0; it < kIt16; ++it)
            __builtin_nontemporal_store(val[it], (u32x4_t*)(wave_c + (lane_off[it] + (uint32_t)m * band_step)));
          return;
        }
#pragma unroll
        for (int it = 0; it < kIt16; ++it) {
          const int e = it * 64 + slane;
          const int r = e / CH, q = e % CH;
          const int i = row0 + wm * Cfg::WTM + m * 16 + r;
          const int j = col0 + wn * Cfg::WTN + q * 8;
          if (i < pe.M && j < pe.N) {
            TO* c = Cb + (int64_t)i * pe.ldc + j;
            if (j + 8 <= pe.N) {
              __builtin_nontemporal_store(val[it], (u32x4_t*)c);   // C is not read again here: keep it from displacing A and B in L2
            } else {                               // ragged right edge: element by element
#pragma unroll
              for (int t2 = 0; t2 < 8; ++t2) {
                const uint32_t word = val[it][t2 >> 1];
                const uint16_t h = (t2 & 1) ? (uint16_t)(word >> 16) : (uint16_t)(word & 0xffffu);
                if (j + t2 < pe.N) ((uint16_t*)c)[t2] = h;
              }
            }
          }
        }
      };
      values(std::integral_constant<int, 0>());
      static_for<0, MT>([&](auto m_c) __attribute__((always_inline)) {
        constexpr int m = decltype(m_c)::value;
        write(m & 1);
        if constexpr (m > 0) read((m - 1) & 1);
        if constexpr (m + 1 < MT) values(std::integral_constant<int, m + 1>());
        if constexpr (m > 0) store(m - 1);
      });
      read((MT - 1) & 1);
      store(MT - 1);
    };
    // fp32 through LDS, one band at a time (one staging buffer: a band is twice the bytes)
    auto drain32_all = [&](auto actf) __attribute__((always_inline)) {
      float* Cf = (float*)pe.C + (int64_t)batch * pe.stride_c;
      const int slane = fresh_lane();
      constexpr int kIt32 = 16 * CH32 / 64;
      const bool inside = row0 + BM <= pe.M && col0 + BN <= pe.N && (int64_t)BM * pe.ldc * 4 < ((int64_t)1 << 31);
      char* const wave_c = (char*)(Cf + (int64_t)(row0 + wm * Cfg::WTM) * pe.ldc + col0 + wn * Cfg::WTN);
      const uint32_t band_step = (uint32_t)(16 * pe.ldc * 4);
      uint32_t lane_off[kIt32];
#pragma unroll
      for (int it = 0; it < kIt32; ++it) {
        const int e = it * 64 + slane;
        lane_off[it] = (uint32_t)((e / CH32) * (int)pe.ldc * 4 + (e % CH32) * 16);
      }
      static_for<0, MT>([&](auto m_c) __attribute__((always_inline)) {
        constexpr int m = decltype(m_c)::value;
#pragma unroll
        for (int n = 0; n < NT; ++n) {
          float bv[4];
          bias4(col0 + wn * Cfg::WTN + n * 16 + eq * 4, bv);
          f32x4_t w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = actf(acc[m][n][e] + bv[e]);
          const int q = n * 4 + eq;
          *(f32x4_t*)(wt + er * OROWB32 + ((q ^ (er & 15)) * 16)) = w;
        }
#pragma unroll
        for (int it = 0; it < kIt32; ++it) {
          const int e = it * 64 + slane;
          const int r = e / CH32, q = e % CH32;
          const f32x4_t val = *(const f32x4_t*)(wt + r * OROWB32 + ((q ^ (r & 15)) * 16));
          if (inside) {
            f32x4_t* c = (f32x4_t*)(wave_c + (lane_off[it] + (uint32_t)m * band_step));
            if (pe.c_cached) *c = val;             // split-K partials are read by the next kernel
            else __builtin_nontemporal_store(val, c);
            continue;
          }
          const int i = row0 + wm * Cfg::WTM + m * 16 + r;
          const int j = col0 + wn * Cfg::WTN + q * 4;
          if (i < pe.M && j < pe.N) {
            float* c = Cf + (int64_t)i * pe.ldc + j;
            if (j + 4 <= pe.N) {
              if (pe.c_cached) *(f32x4_t*)c = val;
              else __builtin_nontemporal_store(val, (f32x4_t*)c);
            } else {
#pragma unroll
              for (int t2 = 0; t2 < 4; ++t2)
                if (j + t2 < pe.N) c[t2] = val[t2];
            }
          }
        }
      });
    };
    // straight from the accumulator layout (C rows that are not 16-byte aligned)
    auto drain = [&](auto actf) __attribute__((always_inline)) {
      const bool vec_ok = (pe.ldc % 4 == 0) && (((uintptr_t)pe.C & 15) == 0) && (pe.stride_c % 4 == 0);
#pragma unroll
      for (int n = 0; n < NT; ++n) {
        const int j = col0 + wn * Cfg::WTN + n * 16 + eq * 4;
        float bv[4];
        bias4(j, bv);
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = actf(acc[m][n][e] + bv[e]);
          const int i = row0 + wm * Cfg::WTM + m * 16 + er;
          if (i >= pe.M || j >= pe.N) continue;
          const bool full = (j + 3 < pe.N);
          const int64_t o = (int64_t)batch * pe.stride_c + (int64_t)i * pe.ldc + j;
          if (pe.c_f32) {
            float* c = (float*)pe.C + o;
            if (full && vec_ok) {
              f32x4_t w = {v[0], v[1], v[2], v[3]};
              *(f32x4_t*)c = w;
            } else {
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (j + e < pe.N) c[e] = v[e];
            }
          } else {
            TO* c = (TO*)pe.C + o;
            if (full && vec_ok) {
              u32x2_t w = {pack2<TO>(v[0], v[1]), pack2<TO>(v[2], v[3])};
              *(u32x2_t*)c = w;
            } else {
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (j + e < pe.N) c[e] = from_float<TO>(v[e]);
            }
          }
        }
      }
    };
    // dest: 0 = memory from the accumulator layout, 1 = 16-bit through LDS, 2 = fp32 through LDS
    auto drain_to = [&](auto actf, auto dest) __attribute__((always_inline)) {
      constexpr int kDest = decltype(dest)::value;
      if constexpr (kDest == 2) {
        drain32_all(actf);
      } else if constexpr (kDest == 1) {
        drain16_all(actf);
      } else {
        drain(actf);
      }
    };
    auto drain_by_activation = [&](auto dest) __attribute__((always_inline)) {
      switch (act) {
        case kActRelu: drain_to([](float x) { return fmaxf(x, 0.0f); }, dest); break;
        case kActGeluErf: drain_to([](float x) { return gelu_erf_f32(x); }, dest); break;
        case kActGeluTanh: drain_to([](float x) { return gelu_tanh_f32(x); }, dest); break;
        case kActSwishScale: { const float c = pe.scale; drain_to([c](float x) { return swish_scale_f32(x, c); }, dest); } break;
        case kActSigmoidScaleResidual: { const float c = pe.scale; drain_to([c](float x) { return sigmoid_scale_residual_f32(x, c); }, dest); } break;
        default: drain_to([](float x) { return x; }, dest); break;
      }
    };

    if (!through_lds && !through_lds32) {
      // (a persistent workgroup is only launched for C rows that take the staged routes below)
      if constexpr (!PERSIST) drain_by_activation(std::integral_constant<int, 0>());
      return;
    }
    if constexpr (!PERSIST) {
      __builtin_amdgcn_s_barrier();              // all waves are done reading the slab stages
      asm volatile("" ::: "memory");
    }
    if (through_lds32) {
      drain_by_activation(std::integral_constant<int, 2>());
      return;
    }
    drain_by_activation(std::integral_constant<int, 1>());
  };

  // ---- main loop ------------------------------------------------------------------------
  // Slab t lives in LDS stage t % 2.  The hand-over to slab t+1 (own reads retired, own loads
  // landed, all waves met) sits before the last sub-step of slab t, whose fragments are
  // already in registers; stage t % 2 is free from then on and is refilled with slab t+2 over
  // the next LW sub-steps (the last one of slab t and the first ones of slab t+1), which
  // leaves the remaining sub-steps before the next hand-over for the loads to land.
  // Priorities (two waves per SIMD): highest right after the hand-over, one lower per
  // sub-step, so the wave that is behind runs first.
  const int T_full = p.K / BK;
  constexpr int LW = NSUB >= 4 ? NSUB - 1 : 1;           // sub-steps the loads of a slab are spread over
  int stage = 0, t = 0;
  SlabIo io_none{nullptr, nullptr, 0u, 0u};
  // early: the rest of the loads of slab t+1 (begun after the previous hand-over) into the other
  // stage; late: the first loads of slab t+2 into this stage after the hand-over
  auto slab_body = [&](auto early_c, auto late_c) __attribute__((always_inline)) {
    constexpr bool early = decltype(early_c)::value, late = decltype(late_c)::value;
    SlabIo io_early = io_none, io_late = io_none;
    if constexpr (early) io_early = slab_io(t + 1, stage ^ 1);
    if constexpr (late) io_late = slab_io(t + 2, stage);
    static_for<0, NSUB - 1>([&](auto u_c) __attribute__((always_inline)) {
      constexpr int u = decltype(u_c)::value;
      set_prio(u < 3 ? 2 - u : 0);
      constexpr int q0 = kLoads * (u + 1) / LW, q1 = kLoads * (u + 2) / LW;
      if constexpr (early && u + 1 < LW)
        sub_step(u_c, true, q0 < kLoads ? q0 : kLoads, q1 < kLoads ? q1 : kLoads, io_early);
      else
        sub_step(u_c, true, 0, 0, io_none);
    });
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    set_prio(3);
    flip_read_stage();
    if constexpr (late) sub_step(std::integral_constant<int, NSUB - 1>(), true, 0, kLoads / LW, io_late);
    else sub_step(std::integral_constant<int, NSUB - 1>(), true, 0, 0, io_none);
    stage ^= 1;
  };
  typedef std::integral_constant<bool, true> yes_t;
  typedef std::integral_constant<bool, false> no_t;

  if constexpr (!PERSIST) {
  if (T_full > 0) {
    {
      const SlabIo io0 = slab_io(0, 0);
#pragma unroll
      for (int q = 0; q < kLoads; ++q) issue_one_load(q, io0);
    }
    if (T_full > 1) {
      const SlabIo io1 = slab_io(1, 1);
#pragma unroll
      for (int q = 0; q < kLoads; ++q) issue_one_load(q, io1);
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoads) : "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    read_all(std::integral_constant<int, 0>());
    if (T_full > 2) slab_body(no_t(), yes_t()); else slab_body(no_t(), no_t());
    for (t = 1; t < T_full - 2; ++t) slab_body(yes_t(), yes_t());
    if (T_full >= 3) { slab_body(yes_t(), no_t()); ++t; }
    if (T_full >= 2) { slab_body(no_t(), no_t()); ++t; }
    set_prio(0);
    // the last fragment reads (of a stage nobody multiplies) are still in flight
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    if (stage) flip_read_stage();              // the K tail reads stage 0
  }
  if (T_full * BK < p.K) {                     // K tail, through registers with zero fill
    __builtin_amdgcn_s_barrier();              // every wave is done with the LDS stages
    asm volatile("" ::: "memory");
    issue_loads_tail(T_full, 0);
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const int ksteps = (p.K - T_full * BK + 31) / 32;
    static_for<0, NSUB>([&](auto u_c) __attribute__((always_inline)) {
      constexpr int u = decltype(u_c)::value;
      if (u / G < ksteps) {
        read_all(u_c);
        sub_step(u_c, false, 0, 0, io_none);
      }
    });
    wait_lgkmcnt<0>();
  }
  int tm, tn;
  tile_coords(p, blockIdx.x, n_tiles, tm, tn);
  epilogue(tm * BM, tn * BN);
  } else {
  // ---- persistent: the tiles of this workgroup as one stream of slabs ------------------------
  // The loads run two slabs ahead of the MFMAs and simply carry on into the next tile's panels:
  // every slab body but the last two of the last tile requests loads.  ld_a / ld_b and the lane
  // offsets describe the slab the loads are at; they move on one slab at a time and switch to
  // the next tile when this one's slabs are all requested.
  int ld_vid = blockIdx.x, ld_t = 0;
  auto fresh_lane_id = []() __attribute__((always_inline)) {
    unsigned z = 0;
    asm volatile("" : "+v"(z));
    return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, z));
  };
  auto next_slab = [&]() __attribute__((always_inline)) {
    ld_a += ROWB; ld_b += ROWB;
    if (++ld_t == T_full) {
      ld_t = 0;
      ld_vid += gridDim.x;
      if (ld_vid < total_tiles) load_tile(ld_vid, fresh_lane_id(), 0);   // (no lane id kept in a register across the loop)
    }
  };
  // tile_end (compile time): the last slab of a tile; its last sub-step requests no fragments (the
  // next tile's first ones are read after the epilogue, which then has no fragment registers to
  // keep alive).  early / late (run time; true in every slab but the last two of the last tile):
  // whether the rest of one slab's loads and the first part of the next one's are requested.
  auto body = [&](auto end_c, bool early, bool late) __attribute__((always_inline)) {
    constexpr bool tile_end = decltype(end_c)::value;
    const SlabIo io_early = slab_io_at(ld_a, ld_b, stage ^ 1);
    static_for<0, NSUB - 1>([&](auto u_c) __attribute__((always_inline)) {
      constexpr int u = decltype(u_c)::value;
      set_prio(u < 3 ? 2 - u : 0);
      constexpr int q0 = kLoads * (u + 1) / LW, q1 = kLoads * (u + 2) / LW;
      if constexpr (u + 1 < LW)
        sub_step(u_c, true, q0 < kLoads ? q0 : kLoads, q1 < kLoads ? q1 : kLoads, io_early, early);
      else
        sub_step(u_c, true, 0, 0, io_none);
    });
    if (late) next_slab();                     // the early part was the rest of a slab: on to the next one
    const SlabIo io_late = slab_io_at(ld_a, ld_b, stage);
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    set_prio(3);
    flip_read_stage();
    sub_step(std::integral_constant<int, NSUB - 1>(), !tile_end, 0, kLoads / LW, io_late, late);
    stage ^= 1;
  };
  // slab 0 whole and the first part of slab 1; from then on every body requests the rest of one
  // slab and the first part of the next
  {
    const SlabIo io0 = slab_io_at(ld_a, ld_b, 0);
#pragma unroll
    for (int q = 0; q < kLoads; ++q) issue_one_load(q, io0);
    next_slab();
    const SlabIo io1 = slab_io_at(ld_a, ld_b, 1);
#pragma unroll
    for (int q = 0; q < kLoads / LW; ++q) issue_one_load(q, io1);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoads / LW) : "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  }
  for (int vid = blockIdx.x; vid < total_tiles; vid += gridDim.x) {
    const bool last = vid + (int)gridDim.x >= total_tiles;
    read_all(std::integral_constant<int, 0>());
    for (t = 0; t < T_full - 2; ++t) body(no_t(), true, true);
    body(no_t(), true, !last);
    body(yes_t(), !last, !last);
    set_prio(0);
    wait_lgkmcnt<0>();
    int tm, tn;
    const int lid = logical_tile(vid);
    batch = lid / n_tiles;
    tile_coords(p, lid - batch * n_tiles, n_tiles, tm, tn);
    epilogue(tm * BM, tn * BN);
    if (!last) {
      // the lane-dependent offsets and addresses are derived afresh here (from an opaque copy of the
      // lane id, so that the compiler cannot keep the earlier ones alive across the epilogue instead)
      const int lane_now = fresh_lane_id();
      load_tile(ld_vid, lane_now, ld_t);
      set_read_stage(stage, lane_now);
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n)
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[m][n][r] = 0.0f;
      // (the next MFMAs are assembly statements the compiler's hazard recogniser cannot see: give the
      // accumulator writes above time to retire, and keep them above this point)
#pragma unroll
      for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int n = 0; n < NT; ++n) asm volatile("" : "+a"(acc[m][n]));
      asm volatile("s_nop 7" ::: "memory");
    }
  }
  }
}

}  // namespace mi355gemm
