// Matrix-core GEMM for gfx950: 16-bit operands (bf16 / fp16) or 8-bit floating point
// (OCP E4M3), fp32 accumulate.
//
//   C = act(A . B + bias),  A row-major (K contiguous), B column-major (K
//   contiguous: the "weight" matrix stored N x K), C row-major.
//
// One workgroup of WM x WN wavefronts owns a BM x BN block of C.  Per K-step of
// BK columns the A and B slabs go global -> LDS with 16-byte direct-to-LDS
// loads (no VGPR staging), NSTAGE slabs deep; wavefronts read MFMA fragments
// with 16-byte LDS reads from an XOR-swizzled layout and issue
// v_mfma_f32_32x32x16 on a (BM/WM) x (BN/WN) register block of accumulators.
// The epilogue (bias, activation, rounding) runs on the accumulators in
// registers.  Paper taxonomy (Sec. 3.2): d_mem = 3 (local-memory tiling +
// register blocking + prefetch), d_algo = 1 (fused post-op), d_sync = 1.
#pragma once

#include <type_traits>

#include "common.hpp"

namespace mi355gemm {

struct MfmaArgs {
  const void* A; const void* B; void* C; const float* bias;
  int M, N, K;
  int64_t lda, ldb, ldc;                               // elements
  int64_t stride_a, stride_b, stride_c, stride_bias;   // elements between batches
  int has_bias, act, c_f32;
  float scale;                 // scalar of the *_scale activations
  int tiles_m, tiles_n;        // ceil(M/BM), ceil(N/BN)
  int group_m;                 // tile rows per scheduling group
  int xcd_remap;               // 1: spread consecutive tile ids within one XCD; 2 (persistent workgroups, a batch):
                               // consecutive problems of the batch within one XCD
  int c_cached;                // 1: fp32 C is read again right away (split-K partials): ordinary stores
  int batches;                 // problems in the batch (persistent workgroups walk over the tiles of all of them)
};

// ---- MFMA wrappers -----------------------------------------------------------
template <typename T> struct Frag;
// Issued through inline assembly: the accumulators are pinned to the AccVGPR file
// ("+a") and, being volatile, the MFMAs keep their program order relative to each
// other and to the (volatile) fragment reads, which is what the hand-made
// software pipeline below relies on.
// A fragment is kParts 16-byte LDS reads per lane: one for the 16-bit types (8 values of K
// per lane and MFMA), two for fp8, whose v_mfma_f32_32x32x64_f8f6f4 takes 32 values of K per
// lane (lane l: row l % 32; which 32 values of the step's 64 a lane holds is free as long
// as A and B agree, so the two reads are the same pair of adjacent 16-byte chunks that two
// consecutive 16-bit steps would read).  kKStep = values of K one MFMA consumes.
template <> struct Frag<bf16_t> {
  static constexpr int kParts = 1, kKStep = 16;
  static __device__ __forceinline__ void mfma(const u32x4_t (&x)[1], const u32x4_t (&y)[1], f32x16_t& c) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(c) : "v"(x[0]), "v"(y[0]));
  }
};
template <> struct Frag<f16_t> {
  static constexpr int kParts = 1, kKStep = 16;
  static __device__ __forceinline__ void mfma(const u32x4_t (&x)[1], const u32x4_t (&y)[1], f32x16_t& c) {
    asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(c) : "v"(x[0]), "v"(y[0]));
  }
};
template <> struct Frag<f8e4m3_t> {
  static constexpr int kParts = 2, kKStep = 64;
  static __device__ __forceinline__ void mfma(const u32x4_t (&x)[2], const u32x4_t (&y)[2], f32x16_t& c) {
    typedef int i32x4_t __attribute__((ext_vector_type(4)));
    typedef int i32x8_t __attribute__((ext_vector_type(8)));
    const i32x8_t xv = __builtin_shufflevector(__builtin_bit_cast(i32x4_t, x[0]), __builtin_bit_cast(i32x4_t, x[1]),
                                               0, 1, 2, 3, 4, 5, 6, 7);
    const i32x8_t yv = __builtin_shufflevector(__builtin_bit_cast(i32x4_t, y[0]), __builtin_bit_cast(i32x4_t, y[1]),
                                               0, 1, 2, 3, 4, 5, 6, 7);
    // both operand formats default to fp8 E4M3, no block scaling
    asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, %0" : "+a"(c) : "v"(xv), "v"(yv));
  }
};

// ---- LDS layout ------------------------------------------------------------------
// A slab is rows x BK values, i.e. rows of 2*HB bytes = HB/8 chunks of 16 bytes (HB = BK
// for the 16-bit types, BK/2 for fp8).  Chunk c of row r is stored at chunk slot
// r*(HB/8) + (c ^ swz<HB>(r)):  the XOR spreads the 32 rows a fragment read touches over
// all LDS banks.
template <int HB> __device__ __forceinline__ int swz(int r);
template <> __device__ __forceinline__ int swz<64>(int r) { return (r & 7) ^ ((r >> 3) & 3); }
template <> __device__ __forceinline__ int swz<32>(int r) {
  return ((r >> 1) & 3) ^ ((r >> 3) & 1);
}

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(3))) unsigned char lds_uchar_t;

// 16-byte LDS read, asynchronous: the destination is valid only after a matching
// s_waitcnt lgkmcnt.  Issued through volatile inline assembly so that reads and
// MFMAs keep exactly their program order; the waits are placed by hand (the
// compiler does not track these reads).
template <typename F>
__device__ __forceinline__ void lds_read_b128(F& dst, uint32_t addr, int offset) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(offset) : "memory");
}
template <int N> __device__ __forceinline__ void wait_lgkmcnt() {
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}
// `n` is a constant after unrolling; the switch turns it into an immediate.
__device__ __forceinline__ void wait_lgkmcnt_dyn(int n) {
  switch (n) {
    case 0: wait_lgkmcnt<0>(); break;   case 1: wait_lgkmcnt<1>(); break;
    case 2: wait_lgkmcnt<2>(); break;   case 3: wait_lgkmcnt<3>(); break;
    case 4: wait_lgkmcnt<4>(); break;   case 5: wait_lgkmcnt<5>(); break;
    case 6: wait_lgkmcnt<6>(); break;   case 7: wait_lgkmcnt<7>(); break;
    case 8: wait_lgkmcnt<8>(); break;   case 9: wait_lgkmcnt<9>(); break;
    case 10: wait_lgkmcnt<10>(); break; case 11: wait_lgkmcnt<11>(); break;
    case 12: wait_lgkmcnt<12>(); break; case 13: wait_lgkmcnt<13>(); break;
    case 14: wait_lgkmcnt<14>(); break; default: wait_lgkmcnt<15>(); break;
  }
}
typedef __attribute__((address_space(1))) const void global_cvoid_t;

__device__ __forceinline__ void wait_vmcnt_0() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// ---- tile scheduling -------------------------------------------------------------
// Workgroups are handed to the 8 XCDs round-robin; each XCD has its own L2.
// Re-number so that each XCD works through one contiguous run of tile ids, and
// walk the tile grid in groups of `group_m` tile rows so that concurrently
// running workgroups share A row-panels and B column-panels in that L2.
__device__ __forceinline__ void tile_coords(const MfmaArgs& p, int wg, int n_wg,
                                            int& tm, int& tn) {
  int id = wg;
  if (p.xcd_remap == 1) {
    const int per = n_wg >> 3;                 // n_wg is a multiple of 8 when remap is on
    id = (wg & 7) * per + (wg >> 3);
  }
  const int in_group = p.group_m * p.tiles_n;
  const int g = id / in_group;
  const int first_m = g * p.group_m;
  const int rows = min(p.tiles_m - first_m, p.group_m);
  const int rem = id - g * in_group;
  tm = first_m + rem % rows;
  tn = rem / rows;
}

// ---- instruction order of one MFMA k-step -----------------------------------------
// A wave block of MT x NT MFMA tiles needs MT A-fragments and NT B-fragments per
// k-step.  Reads are requested in the order a0 b0 b1 a1 b2 a2 ...; the MFMAs run in
// the order in which both of their operands have been requested.
template <int MT, int NT>
struct StepOrder {
  static constexpr int kReads = MT + NT, kMfma = MT * NT;
  struct Tables {
    int r_isb[kReads], r_idx[kReads];
    int mm[kMfma], nn[kMfma];
    int need[kMfma];        // request position of the later of MFMA i's two operands
  };
  static constexpr Tables make() {
    Tables t{};
    int pos_a[MT] = {}, pos_b[NT] = {};
    int c = 0;
    for (int i = 0; i < (MT > NT ? MT : NT); ++i) {
      if (i == 0) {
        t.r_isb[c] = 0; t.r_idx[c] = 0; pos_a[0] = c++;
        t.r_isb[c] = 1; t.r_idx[c] = 0; pos_b[0] = c++;
      } else {
        if (i < NT) { t.r_isb[c] = 1; t.r_idx[c] = i; pos_b[i] = c++; }
        if (i < MT) { t.r_isb[c] = 0; t.r_idx[c] = i; pos_a[i] = c++; }
      }
    }
    // selection sort of the (m, n) pairs by the later of their two request positions
    bool used[kMfma] = {};
    for (int i = 0; i < kMfma; ++i) {
      int best = -1, best_key = 0;
      for (int q = 0; q < kMfma; ++q) {
        if (used[q]) continue;
        const int m = q / NT, n = q % NT;
        const int key = (pos_a[m] > pos_b[n] ? pos_a[m] : pos_b[n]) * kMfma + q;
        if (best < 0 || key < best_key) { best = q; best_key = key; }
      }
      used[best] = true;
      t.mm[i] = best / NT;
      t.nn[i] = best % NT;
      t.need[i] = best_key / kMfma;
    }
    return t;
  }
  static constexpr Tables t = make();
};

template <typename T, int BM, int BN, int BK, int WM, int WN, int NSTAGE>
struct MfmaTile {
  static constexpr int kThreads = 64 * WM * WN;
  static constexpr int kWaves = WM * WN;
  static constexpr int WTM = BM / WM, WTN = BN / WN;     // per-wave block
  static constexpr int MT = WTM / 32, NT = WTN / 32;     // 32x32 MFMA tiles per wave
  static constexpr int ES = (int)sizeof(T);              // bytes per operand element
  static constexpr int EPC = 16 / ES;                    // elements per 16-byte chunk
  static constexpr int ROWB = BK * ES;                   // bytes per slab row
  static constexpr int HB = ROWB / 2;                    // key of the swizzle
  static constexpr int CPR = ROWB / 16;                  // 16-byte chunks per slab row
  static constexpr int RPI = 64 / CPR;                   // slab rows one wave-wide load covers
  static constexpr int A_LOADS = BM / RPI / kWaves;      // direct-to-LDS loads per lane, A slab
  static constexpr int B_LOADS = BN / RPI / kWaves;
  static constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB;
  static constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
  static constexpr int KK = BK / Frag<T>::kKStep;        // MFMA k-steps per slab
  static_assert(BM % (RPI * kWaves) == 0 && BN % (RPI * kWaves) == 0, "slab rows must divide over waves");
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave block must be a multiple of 32x32");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
  static_assert(NSTAGE >= 2, "the hand-over waits assume at least two stages");
  static_assert(MT * NT >= MT + NT, "a k-step issues one fragment read behind each MFMA: it needs at least as "
                                    "many MFMAs as reads (wave blocks of at least 2 x 2 MFMA tiles)");
};

// f(integral_constant<int, I>) for I = FROM .. TO-1, unrolled at compile time
template <int FROM, int TO_, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (FROM < TO_) {
    f(std::integral_constant<int, FROM>());
    static_for<FROM + 1, TO_>(f);
  }
}

// T: operand type; TO: the 16-bit output type (outputs may also be fp32: MfmaArgs::c_f32).
template <typename T, typename TO, int BM, int BN, int BK, int WM, int WN, int NSTAGE>
__global__ __launch_bounds__(64 * WM * WN) void mfma_gemm_kernel(MfmaArgs p) {
  typedef MfmaTile<T, BM, BN, BK, WM, WN, NSTAGE> Cfg;
  constexpr int MT = Cfg::MT, NT = Cfg::NT, CPR = Cfg::CPR, RPI = Cfg::RPI;
  constexpr int ES = Cfg::ES, EPC = Cfg::EPC, ROWB = Cfg::ROWB, HB = Cfg::HB;
  constexpr int kParts = Frag<T>::kParts;

  __shared__ __attribute__((aligned(1024))) unsigned char smem[Cfg::LDS_BYTES];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;

  int tm, tn;
  tile_coords(p, blockIdx.x, gridDim.x, tm, tn);
  const int row0 = tm * BM, col0 = tn * BN;
  const int64_t batch = blockIdx.y;

  const T* Ab = (const T*)p.A + batch * p.stride_a + (int64_t)row0 * p.lda;
  const T* Bb = (const T*)p.B + batch * p.stride_b + (int64_t)col0 * p.ldb;

  // ---- global -> LDS addressing -------------------------------------------------
  // Load q of this wave fills LDS bytes [slab + (wave*LOADS + q)*1024, +1024): lane
  // l writes 16 bytes at +16*l, i.e. slab row (wave*LOADS+q)*RPI + l/CPR, slot l%CPR,
  // which must receive logical chunk  slot ^ swz(row).  Rows past the matrix edge
  // are clamped to the last valid row (their results are never stored).
  uint32_t a_off[Cfg::A_LOADS], b_off[Cfg::B_LOADS];
#pragma unroll
  for (int q = 0; q < Cfg::A_LOADS; ++q) {
    const int r = (wave * Cfg::A_LOADS + q) * RPI + lane / CPR;
    const int c = (lane % CPR) ^ swz<HB>(r);
    const int rr = min(r, p.M - 1 - row0);
    a_off[q] = (uint32_t)(((int64_t)rr * p.lda + c * EPC) * ES);
  }
#pragma unroll
  for (int q = 0; q < Cfg::B_LOADS; ++q) {
    const int r = (wave * Cfg::B_LOADS + q) * RPI + lane / CPR;
    const int c = (lane % CPR) ^ swz<HB>(r);
    const int rr = min(r, p.N - 1 - col0);
    b_off[q] = (uint32_t)(((int64_t)rr * p.ldb + c * EPC) * ES);
  }

  // One direct-to-LDS load: q < A_LOADS fills the A slab, the rest the B slab.  Issued as
  // "scalar base + 32-bit lane offset" through inline assembly: the slab's base address is
  // wave-uniform, so no vector ALU work is spent on 64-bit addresses in the MFMA stream.
  // M0 carries the LDS destination of the wave (lane l lands at M0 + 16*l).
  // Every lambda below is forced inline: left to its size heuristics the compiler may keep a
  // call, and with it the captured accumulators and fragments in memory instead of registers,
  // which the hand-placed waits and the assembly statements cannot tolerate.
  const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_uchar_t*)smem;
  auto issue_one_load = [&](int q, int kt, int stage) __attribute__((always_inline)) {
    const bool is_a = q < Cfg::A_LOADS;
    const int qq = is_a ? q : q - Cfg::A_LOADS;
    // (wave-uniform by construction; read back through the scalar unit so that the "s" operand
    // below holds even where the compiler would otherwise carry this address in vector registers)
    const uint64_t gv = (uint64_t)((const char*)(is_a ? Ab : Bb) + (int64_t)kt * ROWB);
    // (the builtin returns a signed int: widen each half as unsigned)
    const uint32_t g_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(gv >> 32));
    const uint32_t g_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)gv);
    const char* g = (const char*)(((uint64_t)g_hi << 32) | (uint64_t)g_lo);
    const uint32_t dst = lds_base + stage * Cfg::STAGE_BYTES + (is_a ? 0 : Cfg::A_BYTES) +
                         (wave * (is_a ? Cfg::A_LOADS : Cfg::B_LOADS) + qq) * 1024;
    const uint32_t off = is_a ? a_off[qq] : b_off[qq];
    // (s_nop 4: where the compiler had to fetch the address from vector registers just before
    // this statement, the load must not read the scalar pair earlier than 5 cycles after that
    // write, and the compiler does not count cycles inside an asm statement; it also covers
    // the one cycle between the M0 write and its use)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 4\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(dst), "v"(off), "s"(g) : "memory", "m0");
  };
  auto issue_loads = [&](int kt, int stage) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < Cfg::A_LOADS + Cfg::B_LOADS; ++q) issue_one_load(q, kt, stage);
  };

  // K tail: the last slab may hold fewer than BK valid columns.  Chunks past K
  // must read as zero, which a direct-to-LDS load cannot do, so that one slab goes
  // through registers.  (K is a multiple of 8: chunks are never split.)
  auto issue_loads_tail = [&](int kt, int stage) __attribute__((always_inline)) {
    const int kvalid = p.K - kt * BK;                      // valid columns in this slab
    const char* ga = (const char*)Ab + (int64_t)kt * ROWB;
    const char* gb = (const char*)Bb + (int64_t)kt * ROWB;
    unsigned char* sa = smem + stage * Cfg::STAGE_BYTES + wave * (Cfg::A_LOADS * 1024);
    unsigned char* sb = smem + stage * Cfg::STAGE_BYTES + Cfg::A_BYTES + wave * (Cfg::B_LOADS * 1024);
#pragma unroll
    for (int q = 0; q < Cfg::A_LOADS; ++q) {
      const int r = (wave * Cfg::A_LOADS + q) * RPI + lane / CPR;
      const int c = (lane % CPR) ^ swz<HB>(r);
      u32x4_t v = {0u, 0u, 0u, 0u};
      if (c * EPC < kvalid) v = *(const u32x4_t*)(ga + a_off[q]);
      *(u32x4_t*)(sa + q * 1024 + lane * 16) = v;
    }
#pragma unroll
    for (int q = 0; q < Cfg::B_LOADS; ++q) {
      const int r = (wave * Cfg::B_LOADS + q) * RPI + lane / CPR;
      const int c = (lane % CPR) ^ swz<HB>(r);
      u32x4_t v = {0u, 0u, 0u, 0u};
      if (c * EPC < kvalid) v = *(const u32x4_t*)(gb + b_off[q]);
      *(u32x4_t*)(sb + q * 1024 + lane * 16) = v;
    }
  };

  // ---- LDS -> fragment addressing -------------------------------------------------
  // MFMA 32x32x16 operand: lane l holds 8 consecutive k of row (l % 32), k-octet l / 32.
  const int fr = lane & 31, fh = lane >> 5;
  const int a_row = wm * Cfg::WTM + fr;
  const int b_row = wn * Cfg::WTN + fr;
  // byte offset of (row, chunk c) = row*ROWB + ((c ^ swz(row)) * 16); part j of k-step kk is
  // chunk (kk*kParts + j)*2 + fh
  uint32_t a_rd[Cfg::KK][kParts], b_rd[Cfg::KK][kParts];
#pragma unroll
  for (int kk = 0; kk < Cfg::KK; ++kk)
#pragma unroll
    for (int j = 0; j < kParts; ++j) {
      const int c = (kk * kParts + j) * 2 + fh;
      a_rd[kk][j] = a_row * ROWB + ((c ^ swz<HB>(a_row)) * 16);
      b_rd[kk][j] = Cfg::A_BYTES + b_row * ROWB + ((c ^ swz<HB>(b_row)) * 16);
    }

  f32x16_t acc[MT][NT];
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int n = 0; n < NT; ++n)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[m][n][r] = 0.0f;

  // Fragment registers, double-buffered over the MFMA k-steps of a slab: while the
  // MFMAs of step kk run, the LDS reads of step kk+1 are already in flight.
  u32x4_t af[2][MT][kParts], bf[2][NT][kParts];
  typedef StepOrder<MT, NT> Ord;
  const uint32_t smem_base = lds_base;

  auto read_one = [&](int i, int stage, int kk, int buf) __attribute__((always_inline)) {       // i-th read of the fixed read order
    const uint32_t s = smem_base + stage * Cfg::STAGE_BYTES;
    const int idx = Ord::t.r_idx[i];
#pragma unroll
    for (int j = 0; j < kParts; ++j) {
      if (Ord::t.r_isb[i]) lds_read_b128(bf[buf][idx][j], s + b_rd[kk][j], idx * (32 * ROWB));
      else lds_read_b128(af[buf][idx][j], s + a_rd[kk][j], idx * (32 * ROWB));
    }
  };
  auto read_frags = [&](int stage, int kk, int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < Ord::kReads; ++i) read_one(i, stage, kk, buf);
  };

  // One MFMA k-step on fragment buffer `cur`, instruction order pinned.  The wave
  // issues in order (and, in the 4-wave shapes, alone on its SIMD), so a wait costs
  // MFMA time: the reads for the next step (slab stage `rs`, k-step `rk`) go out one
  // behind each of the first MFMAs, first-needed operands first, and the MFMAs run in
  // the order in which their operands were requested one step earlier, so that every
  // read has almost a whole step to land.  With `loads`, the direct-to-LDS loads of
  // slab `lk` into stage `ls` follow the reads, spread over the remaining MFMAs.
  // Operands go in swapped (B fragment first) so that a lane ends up holding one row
  // of C and runs of 4 consecutive columns: that is what the stores want.
  auto step = [&](int cur, bool reads, int rs, int rk, bool loads, int lk, int ls) __attribute__((always_inline)) {
    constexpr int kLoads = Cfg::A_LOADS + Cfg::B_LOADS;
    constexpr int kLeft = Ord::kMfma;
    constexpr int kPer = (kLoads + kLeft - 1) / kLeft;
#pragma unroll
    for (int i = 0; i < Ord::kMfma; ++i) {
      const int m = Ord::t.mm[i], n = Ord::t.nn[i];
      // LDS reads return in order: the operands of MFMA i were requested at position
      // need[i] of the previous step's kReads requests; since then the rest of those
      // and min(i, kReads) requests of this step have been issued.
      {
        const int after = (Ord::kReads - 1 - Ord::t.need[i]) + (reads ? (i < Ord::kReads ? i : Ord::kReads) : 0);
        wait_lgkmcnt_dyn(after * kParts);        // (the counter holds 15 at most: larger values wait for 15)
      }
      Frag<T>::mfma(bf[cur][n], af[cur][m], acc[m][n]);
      if (reads && i < Ord::kReads) read_one(i, rs, rk, cur ^ 1);
      if (loads) {
        const int j = i;
        if (j >= 0) {
#pragma unroll
          for (int q = j * kPer; q < (j + 1) * kPer && q < kLoads; ++q) issue_one_load(q, lk, ls);
        }
      }
    }
  };

  // ---- main loop ------------------------------------------------------------------
  // Full slabs (all BK columns valid) 0 .. T_full-1 run through a branch-free loop;
  // slab t lives in LDS stage t % NSTAGE.  The hand-over to slab t+1 happens before
  // the last MFMA step of slab t (whose fragments are already in registers), so the
  // barrier and the first fragment reads of slab t+1 hide behind those MFMAs, and
  // stage t % NSTAGE is refilled with slab t+NSTAGE right after the barrier.  Every
  // iteration of that loop issues the same number of loads, so the wait counts are
  // constants and the body has no branch in it; the last NSTAGE slabs, which have nothing
  // left to prefetch, run through a second copy of the body without loads that waits for
  // everything outstanding.  A K tail (K % BK != 0) is multiplied after the loops.
  const int T_full = p.K / BK;
  constexpr int kLoadsPerSlab = Cfg::A_LOADS + Cfg::B_LOADS;
  constexpr int D = NSTAGE;                    // prefetch distance in slabs
  constexpr int KK = Cfg::KK;
  static_assert(KK % 2 == 0, "fragment double buffer assumes an even number of k-steps");

  // Own LDS reads retired (the stage may be refilled) and own loads of the wanted
  // slab landed, the loads of `kLater` later slabs may stay in flight; then all
  // waves meet.
  auto hand_over = [&](auto later) __attribute__((always_inline)) {
    constexpr int kLater = decltype(later)::value;
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(kLater * kLoadsPerSlab) : "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    // Two waves share a SIMD: the one that has just passed the hand-over runs its last k-step (and
    // issues the refill) at high priority, then drops; the wave that is behind gets the matrix pipe.
    if (Cfg::kWaves > 4) asm volatile("s_setprio 3" ::: "memory");
  };
  auto drop_prio = [&]() __attribute__((always_inline)) {
    if (Cfg::kWaves > 4) asm volatile("s_setprio 0" ::: "memory");
  };

  if (T_full > 0) {
#pragma unroll
    for (int s = 0; s < D; ++s) issue_loads(min(s, T_full - 1), s);
    hand_over(std::integral_constant<int, D - 1>());
    read_frags(0, 0, 0);
    int stage = 0;
    int t = 0;
    for (; t < T_full - D; ++t) {              // slab t + D exists: refill the stage just freed
      const int next_stage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
#pragma unroll
      for (int kk = 0; kk < KK - 1; ++kk) step(kk & 1, true, stage, kk + 1, false, 0, 0);
      hand_over(std::integral_constant<int, D - 2>());
      // (min: t + D <= T_full - 1 here; written out, it keeps the slab address in scalar registers)
      step((KK - 1) & 1, true, next_stage, 0, true, min(t + D, T_full - 1), stage);
      drop_prio();
      stage = next_stage;
    }
    for (; t < T_full; ++t) {                  // the last D slabs: nothing left to prefetch
      const int next_stage = (stage + 1 == NSTAGE) ? 0 : stage + 1;
#pragma unroll
      for (int kk = 0; kk < KK - 1; ++kk) step(kk & 1, true, stage, kk + 1, false, 0, 0);
      hand_over(std::integral_constant<int, 0>());
      step((KK - 1) & 1, true, next_stage, 0, false, 0, 0);
      drop_prio();
      stage = next_stage;
    }
    // the last fragment reads (of a stage nobody multiplies) are still in flight
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  }
  if (T_full * BK < p.K) {                     // K tail, through registers with zero fill
    __builtin_amdgcn_s_barrier();              // every wave is done with the LDS stages
    asm volatile("" ::: "memory");
    issue_loads_tail(T_full, 0);
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    const int ksteps = (p.K - T_full * BK + Frag<T>::kKStep - 1) / Frag<T>::kKStep;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      if (kk < ksteps) {
        // alternate the fragment buffers as the main loop does: a step's reads must not land
        // in registers that MFMAs of the step before, still queued, have yet to read
        read_frags(0, kk, kk & 1);
        step(kk & 1, false, 0, 0, false, 0, 0);
      }
    }
    wait_lgkmcnt<0>();
  }

  // The MFMAs were issued through inline assembly, so the compiler does not know that the
  // accumulators are matrix-core results and inserts none of the wait states a vector-ALU
  // read of a just-written MFMA result needs (there is no hardware interlock: up to 19
  // cycles after a 16-pass instruction).  Wait once, and route every accumulator through an
  // (empty) volatile statement placed after the wait, so that no read can be scheduled
  // above it.  Without this the last k-step of a K tail was lost for the MFMA tiles issued
  // last whenever nothing else separated it from the epilogue.
  asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");
#pragma unroll
  for (int m = 0; m < MT; ++m)
#pragma unroll
    for (int n = 0; n < NT; ++n) asm volatile("" : "+a"(acc[m][n]));

  // ---- epilogue ---------------------------------------------------------------------
  // Lane l of a 32x32 accumulator tile holds row (l % 32) and, in register r,
  // column 8*(r/4) + 4*(l/32) + r%4: runs of only 4 columns per lane.  Storing those
  // directly makes every store instruction touch 64 different cache lines with 8 or 16
  // bytes each.  For 16-bit output each wave therefore passes its block through its
  // own piece of the (now idle) LDS: 8-byte writes in accumulator order, 16-byte reads
  // in row order, and the global stores cover whole 128-byte lines.
  const float* bias = p.has_bias ? p.bias + batch * p.stride_bias : nullptr;
  const int act = p.act;
  // The lane-dependent addresses of the epilogue are derived from a lane id that is computed
  // afresh where it is needed (from an opaque zero, so that the compiler can neither hoist it
  // above the K loop nor keep one copy alive across the accumulator reads): the K loop and
  // the drain have no register to spare for them.  (All 64 lanes are active here.)
  auto fresh_lane = []() __attribute__((always_inline)) {
    unsigned z = 0;
    asm volatile("" : "+v"(z));
    return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, z));
  };
  const int elane = fresh_lane();
  const int er = elane & 31, eh = elane >> 5;

  // bias of the 4 columns j .. j+3 (zero past N; j is a multiple of 4); 16-byte loads only when
  // the bias vector of this batch starts at a 16-byte aligned address (the same for every lane)
  const bool bias_vec = (((uintptr_t)bias) & 15) == 0;
  auto bias4 = [&](int j, float (&bv)[4]) __attribute__((always_inline)) {
#pragma unroll
    for (int e = 0; e < 4; ++e) bv[e] = 0.0f;
    if (!bias) return;
    if (j + 3 < p.N && bias_vec) {
      const f32x4_t b4 = *(const f32x4_t*)(bias + j);
#pragma unroll
      for (int e = 0; e < 4; ++e) bv[e] = b4[e];
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (j + e < p.N) bv[e] = bias[j + e];
    }
  };

  const bool through_lds = !p.c_f32 && (p.ldc % 8 == 0) && (p.stride_c % 8 == 0) &&
                           (((uintptr_t)p.C & 15) == 0);
  constexpr int OROWB = Cfg::WTN * 2;           // bytes per row of the wave's block
  constexpr int CH = OROWB / 16;                // 16-byte chunks per row (8, 12 or 16)
  constexpr int OSW = CH % 8 == 0 ? 7 : 3;      // chunk-slot swizzle mask: stays inside the row for CH = 12
  static_assert(Cfg::LDS_BYTES >= BM * BN * 2, "the output block must fit the slab stages");
  static_assert(CH >= 8 && CH % 4 == 0 && (32 * CH) % 64 == 0,
                "row of the wave block: at least 128 bytes, and the block a whole number of wave-wide accesses");
  unsigned char* wt = smem + wave * (Cfg::WTM * OROWB);
  // fp32 output goes through the same LDS pieces in passes of MP 32-row tiles (a wave's share of
  // the stages holds a quarter to a half of its block in fp32): 16-byte writes in accumulator
  // order, 16-byte reads in row order, stores that cover whole lines.
  const bool through_lds32 = p.c_f32 && (p.ldc % 4 == 0) && (p.stride_c % 4 == 0) && (((uintptr_t)p.C & 15) == 0);
  constexpr int OROWB32 = Cfg::WTN * 4;         // bytes per fp32 row of the wave's block
  constexpr int CH32 = OROWB32 / 16;            // 16-byte chunks per row (16, 24 or 32)
  constexpr int OSW32 = CH32 % 16 == 0 ? 15 : 7;
  constexpr int kShare = Cfg::LDS_BYTES / Cfg::kWaves;           // bytes of LDS per wave
  constexpr int MP = (kShare / (32 * OROWB32)) >= MT ? MT : (kShare / (32 * OROWB32) >= 2 ? 2 : 1);
  static_assert(32 * OROWB32 <= kShare && MT % MP == 0 && (32 * MP * CH32) % 64 == 0,
                "one 32-row tile of the wave block in fp32 must fit the wave's share of LDS");
  unsigned char* wt32 = smem + wave * kShare;

  // Each accumulator is read once: + bias, activation, rounding, and out (to LDS or
  // to memory).  `actf` and `via_lds` are compile-time: one straight-line copy of the loops
  // per activation and destination (a run-time test per accumulator group costs a taken
  // branch each, which adds up to microseconds per tile).
  // fp32 through LDS: m-tiles [MP pass, MP pass + MP) of every column tile, then their rows out
  auto drain32 = [&](auto actf, auto pass_c) __attribute__((always_inline)) {
    constexpr int pass = decltype(pass_c)::value;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int j = col0 + wn * Cfg::WTN + n * 32 + g * 8 + eh * 4;
        float bv[4];
        bias4(j, bv);
#pragma unroll
        for (int mm = 0; mm < MP; ++mm) {
          const int m = pass * MP + mm;
          f32x4_t w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = actf(acc[m][n][g * 4 + e] + bv[e]);
          const int r = mm * 32 + er, q = n * 8 + g * 2 + eh;
          *(f32x4_t*)(wt32 + r * OROWB32 + ((q ^ (r & OSW32)) * 16)) = w;
        }
      }
    }
    float* Cf = (float*)p.C + batch * p.stride_c;
    const int slane32 = fresh_lane();
#pragma unroll
    for (int it = 0; it < 32 * MP * CH32 / 64; ++it) {
      const int e = it * 64 + slane32;
      const int r = e / CH32, q = e % CH32;
      const f32x4_t val = *(const f32x4_t*)(wt32 + r * OROWB32 + ((q ^ (r & OSW32)) * 16));
      const int i = row0 + wm * Cfg::WTM + pass * (32 * MP) + r;
      const int j = col0 + wn * Cfg::WTN + q * 4;
      if (i < p.M && j < p.N) {
        float* c = Cf + (int64_t)i * p.ldc + j;
        if (j + 4 <= p.N) {
          // C is normally not read again here: non-temporal, so that it does not displace A and B
          // in L2; split-K partials are read by the next kernel and should stay cached
          if (p.c_cached) *(f32x4_t*)c = val;
          else __builtin_nontemporal_store(val, (f32x4_t*)c);
        } else {
#pragma unroll
          for (int t = 0; t < 4; ++t)
            if (j + t < p.N) c[t] = val[t];
        }
      }
    }
  };
  // 16-bit through LDS, one 32-row tile of the wave block per pass: its rows are on their way
  // to memory while the next tile's accumulators are drained
  auto drain16 = [&](auto actf, auto pass_c) __attribute__((always_inline)) {
    constexpr int m = decltype(pass_c)::value;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int j = col0 + wn * Cfg::WTN + n * 32 + g * 8 + eh * 4;
        float bv[4];
        bias4(j, bv);
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = actf(acc[m][n][g * 4 + e] + bv[e]);
        // chunk q of row r sits at chunk slot q ^ ((r >> 1) & OSW): spreads the 32 rows
        // a write instruction touches over the banks
        const int r = m * 32 + er, q = n * 4 + g;
        u32x2_t w = {pack2<TO>(v[0], v[1]), pack2<TO>(v[2], v[3])};
        *(u32x2_t*)(wt + r * OROWB + ((q ^ ((r >> 1) & OSW)) * 16) + eh * 8) = w;
      }
    }
    TO* Cb = (TO*)p.C + batch * p.stride_c;
    const int slane = fresh_lane();
#pragma unroll
    for (int it = 0; it < 32 * CH / 64; ++it) {
      // the tile's 16-byte chunks in row-major order, 64 per access: whole rows (or runs of rows)
      const int e = it * 64 + slane;
      const int r = m * 32 + e / CH, q = e % CH;
      const u32x4_t val = *(const u32x4_t*)(wt + r * OROWB + ((q ^ ((r >> 1) & OSW)) * 16));
      const int i = row0 + wm * Cfg::WTM + r;
      const int j = col0 + wn * Cfg::WTN + q * 8;
      if (i < p.M && j < p.N) {
        TO* c = Cb + (int64_t)i * p.ldc + j;
        if (j + 8 <= p.N) {
          __builtin_nontemporal_store(val, (u32x4_t*)c);   // C is not read again here: keep it from displacing A and B in L2
        } else {                                 // ragged right edge: element by element
#pragma unroll
          for (int t = 0; t < 8; ++t) {
            const uint32_t word = val[t >> 1];
            const uint16_t h = (t & 1) ? (uint16_t)(word >> 16) : (uint16_t)(word & 0xffffu);
            if (j + t < p.N) ((uint16_t*)c)[t] = h;
          }
        }
      }
    }
  };
  // straight from the accumulator layout (C rows that are not 16-byte aligned)
  auto drain = [&](auto actf) __attribute__((always_inline)) {
    const bool vec_ok = (p.ldc % 4 == 0) && (((uintptr_t)p.C & 15) == 0) && (p.stride_c % 4 == 0);
#pragma unroll
    for (int n = 0; n < NT; ++n) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int j = col0 + wn * Cfg::WTN + n * 32 + g * 8 + eh * 4;
        float bv[4];
        bias4(j, bv);
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = actf(acc[m][n][g * 4 + e] + bv[e]);
          {
            const int i = row0 + wm * Cfg::WTM + m * 32 + er;
            if (i >= p.M || j >= p.N) continue;
            const bool full = (j + 3 < p.N);
            const int64_t o = batch * p.stride_c + (int64_t)i * p.ldc + j;
            if (p.c_f32) {
              float* c = (float*)p.C + o;
              if (full && vec_ok) {
                f32x4_t w = {v[0], v[1], v[2], v[3]};
                *(f32x4_t*)c = w;
              } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                  if (j + e < p.N) c[e] = v[e];
              }
            } else {
              TO* c = (TO*)p.C + o;
              if (full && vec_ok) {
                u32x2_t w = {pack2<TO>(v[0], v[1]), pack2<TO>(v[2], v[3])};
                *(u32x2_t*)c = w;
              } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                  if (j + e < p.N) c[e] = from_float<TO>(v[e]);
              }
            }
          }
        }
      }
    }
  };
  // dest: 0 = memory from the accumulator layout, 1 = 16-bit through LDS, 2 = fp32 through LDS
  auto drain_to = [&](auto actf, auto dest) __attribute__((always_inline)) {
    constexpr int kDest = decltype(dest)::value;
    if constexpr (kDest == 2) {
      static_for<0, MT / MP>([&](auto pass_c) __attribute__((always_inline)) { drain32(actf, pass_c); });
    } else if constexpr (kDest == 1) {
      static_for<0, MT>([&](auto pass_c) __attribute__((always_inline)) { drain16(actf, pass_c); });
    } else {
      drain(actf);
    }
  };
  auto drain_by_activation = [&](auto dest) __attribute__((always_inline)) {
    switch (act) {
      case kActRelu: drain_to([](float t) { return fmaxf(t, 0.0f); }, dest); break;
      case kActGeluErf: drain_to([](float t) { return gelu_erf_f32(t); }, dest); break;
      case kActGeluTanh: drain_to([](float t) { return gelu_tanh_f32(t); }, dest); break;
      case kActSwishScale: { const float c = p.scale; drain_to([c](float t) { return swish_scale_f32(t, c); }, dest); } break;
      case kActSigmoidScaleResidual: { const float c = p.scale; drain_to([c](float t) { return sigmoid_scale_residual_f32(t, c); }, dest); } break;
      default: drain_to([](float t) { return t; }, dest); break;
    }
  };

  if (!through_lds && !through_lds32) {
    drain_by_activation(std::integral_constant<int, 0>());
    return;
  }
  __builtin_amdgcn_s_barrier();                // all waves are done reading the slab stages
  asm volatile("" ::: "memory");
  if (through_lds32) {
    drain_by_activation(std::integral_constant<int, 2>());
    return;
  }
  drain_by_activation(std::integral_constant<int, 1>());
}

}  // namespace mi355gemm
