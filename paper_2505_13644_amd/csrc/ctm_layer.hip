// Stacked GEMM of one MLP layer over the whole coefficient block, with the collapsed
// Taylor-mode rule of the activation fused in as its epilogue (gfx950 MFMA).
//
// What one layer computes (Sec. 3.1, Eq. 6; App. D collapsed scheme):
//   for every point n and every coefficient row c of the point:  z_c = W h_c  (+ b for c = 0),
//   then the activation's Taylor rule on the rows of the point (ctm_rule.h), in which the
//   highest-order row is the one already summed over the directions.
// The same kernel runs the reverse pass: with cotangents as input rows and W transposed it
// computes Hbar = Zbar W and applies the reverse of the rule (order 2 or 4) as its epilogue.
//
// Layout.  The block is point-major: rows n*rho .. n*rho + rho - 1 belong to point n
// (row 0: order 0; then the per-direction rows; last row: the collapsed one), each row
// `ld` elements with zero padding.  A workgroup owns P whole points (P*rho <= 16*MB rows)
// times 64*NB output features, so the sum over directions never leaves the workgroup:
// the accumulators are staged through LDS (64 columns at a time) and each thread then walks
// the rows of one (point, feature) pair, keeping the running sums in registers.
// Registers and LDS per workgroup are kept low enough for two to four workgroups per CU (Tile::kWgPerCu), so that
// one's prologue, epilogue and barriers fall under the MFMAs of the others.  The A and B tiles of a k-block
// reach LDS by LDS-direct loads (no register staging), double-buffered one k-block ahead.
// The same kernel also reverses the order-4 rule (the reverse pass of the randomized / exact biharmonic).
//
// MFMA use: v_mfma_{f32,f64}_16x16x4.  Lane l supplies A[row l%16][k l/16] and
// B[k l/16][col l%16]; it receives four elements of column l%16 of D, in rows
// 4*(l/16) + v for f32 and 4*v + l/16 for f64 (v = register index).  Each lane fetches KV
// consecutive k values with one 16-byte LDS read and feeds them to KV successive MFMAs; since
// A and B use the same assignment, the k-sum is merely taken in a permuted order.
#include "ctm_internal.h"
#include <type_traits>

#include "ctm_rule.h"

namespace ctm {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef double f64x2 __attribute__((ext_vector_type(2)));

template <typename T> struct Vec;
template <> struct Vec<float> {
  using ld = f32x4;   // 16-byte load unit
  using acc = f32x4;  // one 16x16 MFMA block: 4 rows per lane
  static __device__ __forceinline__ int out_row(int lane_group, int v) { return lane_group * 4 + v; }
};
template <> struct Vec<double> {
  using ld = f64x2;
  using acc = f64x4;
  static __device__ __forceinline__ int out_row(int lane_group, int v) { return v * 4 + lane_group; }
};

__device__ __forceinline__ f32x4 mfma16(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f64x4 mfma16(double a, double b, f64x4 c) {
  return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

constexpr int kThreads = 256;
constexpr int kXcds = 8;

template <typename T, int MB> struct Tile {
  static constexpr int KV = Shape<T>::KV;
  static constexpr int BK = Shape<T>::BK;
  static constexpr int NB = Shape<T>::NB;
  static constexpr int BM = 16 * MB;
  static constexpr int BN = 64 * NB;
  static constexpr int PADE = 16 / sizeof(T);     // 16 bytes of padding per row of the staged C chunk
  static constexpr int LROW = BK;                 // LDS row pitch of a stage, elements: 64 bytes, no padding (LDS-direct loads)
  static constexpr int A_STAGE = BM * LROW;
  static constexpr int B_STAGE = BN * LROW;
  static constexpr int CCOLS = 256 / sizeof(T);   // the C tile is staged in two chunks of 256 bytes per row: 64 fp32 / 32 fp64 columns
  // LDS row pitch of the staged C chunk: padded so that the four row groups of an accumulator store hit different
  // banks -- unless the pad is what keeps a third workgroup off the CU (MB = 13 in fp32: 52 KiB without, 55 KiB with)
  static constexpr size_t kCuLds = 160 * 1024;
  static constexpr size_t kStageBytes = 2 * (size_t)(A_STAGE + B_STAGE) * sizeof(T);
  static constexpr bool kDropPad = 3 * (size_t)BM * (CCOLS + PADE) * sizeof(T) > kCuLds && 3 * (size_t)BM * CCOLS * sizeof(T) <= kCuLds &&
                                   3 * kStageBytes <= kCuLds;
  static constexpr int CROW = CCOLS + (kDropPad ? 0 : PADE);
  static constexpr size_t kCBytes = (size_t)BM * CROW * sizeof(T);
  // behind them: the group sums that wavefronts sharing a point hand to the point's first wavefront (two points x 2
  // slots when two wavefronts share a point, one point x 3 slots when four do; 64 columns per slot)
  static constexpr size_t kRedOffset = ((kStageBytes > kCBytes ? kStageBytes : kCBytes) + 15) / 16 * 16;
  static constexpr size_t kRedBytes = 4 * 64 * sizeof(T);   // only allocated by the kernels that share points (WPP > 1)
  // Workgroups per CU the kernel is compiled for (= waves per SIMD: the register budget is 512 / that, rounded down to 8):
  // the accumulators alone take 8 * MB registers (fp32: MB x 2 column blocks x 4; fp64: MB x 1 x 8).
  static constexpr int kWgPerCu = MB <= 9 ? 4 : MB <= 13 ? 3 : 2;
  static constexpr size_t kLdsBytes = kRedOffset + kRedBytes;
  static_assert(BK * sizeof(T) == 64 && BN % 16 == 0, "a 16-row chunk of a stage is one 1 KiB LDS-direct load");
  static_assert(kLdsBytes <= 160 * 1024, "tile does not fit the 160 KiB LDS of a CU");
};

// amdgpu_waves_per_eu caps the registers per lane (4 waves per SIMD: 128, 3: 168, 2: 256).  With a cap the compiler
// keeps the accumulators in ordinary VGPRs and issues MFMAs on them directly; without one (512 registers allowed) it
// parks them in AGPRs and copies each block back and forth around every MFMA group, which left the matrix pipe idle
// almost half of the time.  Three or four resident workgroups instead of two matter because a workgroup spends more
// than half of its life outside the k loop (prologue, epilogue: their vector-ALU instructions only get the issue slots
// the MFMA stream of a co-resident workgroup leaves): the more neighbours, the rarer the moments without MFMAs in flight.
// MODE picks the epilogue at compile time -- one instance per use instead of one kernel with every path in it, which also
// relieves the scalar registers (12 instead of 70 spilled in the plain forward instance; their lane reads and writes are
// vector-ALU instructions):
//   kPlain    forward, collapsed, no tape (what the operator entry points launch)
//   kTape     forward, collapsed, the pre-activation rows are recorded too
//   kReverse  reverse pass: the epilogue is the reverse of the rule
//   kStandard forward in the un-collapsed layout (comparison path)
enum LayerMode { kPlain = 0, kTape = 1, kReverse = 2, kStandard = 3 };
template <typename T, int MB, int WPP, int MODE>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(Tile<T, MB>::kWgPerCu, Tile<T, MB>::kWgPerCu)))
void layer_kernel(const LayerArgs<T> a) {
  using TL = Tile<T, MB>;
  using vld = typename Vec<T>::ld;
  using vacc = typename Vec<T>::acc;
  constexpr int KV = TL::KV, BK = TL::BK, NB = TL::NB, BN = TL::BN;
  constexpr int LROW = TL::LROW, CROW = TL::CROW;

  extern __shared__ __align__(16) unsigned char lds_raw[];
  T *lds = reinterpret_cast<T *>(lds_raw);
  T *As = lds;                      // [2][A_STAGE]
  T *Bs = lds + 2 * TL::A_STAGE;    // [2][B_STAGE]
  T *Cs = lds;                      // [BM][CROW] chunk of the C tile, reuses the stages after the k loop

  // ---- which tile: workgroups are dealt round-robin to the 8 XCDs, each with its own L2.
  // Give every XCD one contiguous run of tiles, ordered so that the column tiles of one
  // row tile (which read the same rows of Hin) are neighbours in time on the same L2.
  // (the launcher keeps the tile count below 2^31, so 32-bit arithmetic does: a 64-bit division is some forty vector-ALU
  // instructions that a starting workgroup would take from its neighbours' MFMAs)
  const unsigned n_tiles = (unsigned)(a.n_row_tiles * a.n_col_tiles);
  const unsigned xcd = blockIdx.x % kXcds;
  const unsigned slot = blockIdx.x / kXcds;
  const unsigned base = n_tiles / kXcds, rem = n_tiles % kXcds;
  const unsigned mine = base + (xcd < rem ? 1 : 0);
  if (slot >= mine) return;
  const unsigned tile = xcd * base + (xcd < rem ? xcd : rem) + slot;
  const long row_tile = tile / (unsigned)a.n_col_tiles;
  const int col_tile = (int)(tile % (unsigned)a.n_col_tiles);

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 15, lg = lane >> 4;

  const long p0 = row_tile * a.P;                                   // first point of the tile
  const int p_valid = (int)((a.n_points - p0) < a.P ? (a.n_points - p0) : a.P);
  const int rows_valid = p_valid * a.rho;                           // <= BM
  const T *Ag = a.Hin + p0 * a.rho * (long)a.ldin;
  const T *Bg = a.W + (long)col_tile * BN * a.ldin;

  // ---- global -> LDS by LDS-direct loads (global_load_lds_dwordx4): every lane names its own 16 global bytes and
  // the wave's 1 KiB lands at LDS address M0 + 16 * lane, without passing through registers.  A stage row is 64 bytes
  // (BK elements, unpadded), so one instruction moves a chunk of 16 rows: lane l brings row l/4 of the chunk, and the
  // row's four 16-byte units are stored XOR-swizzled with bits 1..2 of the row.  Measured on the fragment reads below
  // (16-byte reads, lane l: row l % 16, unit l / 16): with this swizzle the bank-conflict counter reads zero and a wave
  // instruction occupies the LDS for 4 cycles; swizzled with bits 2..3 of the row, or not at all, it took 8 (the hardware
  // serves 8 rows x 2 units per cycle, not 16 rows x 1).  Neutral for this kernel's time: its LDS is idle 85 % of the cycles.  Chunks 0..MB-1 are the A tile, MB..MB+BN/16-1 the
  // B tile; wave w takes chunks w, w+4, ...  Rows past the tile's last valid row re-read that row: they only feed
  // accumulator rows the epilogue never looks at (MFMA rows do not mix).  The loads are unconditional per wave, so
  // the k loop stays branch-free apart from the uniform chunk-count test.
  constexpr int kChunks = MB + BN / 16;
  constexpr int NCH = (kChunks + 3) / 4;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  // Address = uniform tile base (SGPR pair, advanced along k by scalar adds) + per-lane 32-bit byte offset: the k loop
  // issues its loads without a single vector ALU instruction (VALU work there competes with the MFMAs for issue slots;
  // per-lane 64-bit addresses cost 1 % more).
  unsigned c_voff[NCH];  // per-lane byte offset from the operand's tile base (< 2^32: at most 256 rows of ldin elements)
  const T *c_base[NCH];  // uniform: the operand's tile base
  unsigned c_off[NCH];   // byte offset inside buffer 0; buffer 1 adds the stage size of the operand
  unsigned c_step[NCH];  // bytes from buffer 0 to buffer 1 for this chunk's operand
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = wave_u + 4 * i;
    const int rr = lane >> 2;                       // row inside the chunk
    const int uu = (lane & 3) ^ ((rr >> 1) & 3);    // the unit this lane's LDS slot holds
    if (c < MB) {
      const int row = c * 16 + rr;
      const int grow = row < rows_valid ? row : rows_valid - 1;
      c_voff[i] = (unsigned)(((long)grow * a.ldin + uu * KV) * sizeof(T));
      c_base[i] = Ag;
      c_off[i] = (unsigned)(c * 16 * BK * sizeof(T));
      c_step[i] = (unsigned)(TL::A_STAGE * sizeof(T));
    } else {
      const int cb = c < kChunks ? c - MB : 0;
      c_voff[i] = (unsigned)(((long)(cb * 16 + rr) * a.ldin + uu * KV) * sizeof(T));
      c_base[i] = Bg;
      c_off[i] = (unsigned)((2 * TL::A_STAGE + cb * 16 * BK) * sizeof(T));
      c_step[i] = (unsigned)(TL::B_STAGE * sizeof(T));
    }
  }
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)lds_raw;
  auto issue_one = [&](int buf, int k0, int i) {   // i: compile-time after unrolling
    if (wave_u + 4 * i < kChunks) {
      const unsigned off = lds_base + c_off[i] + buf * c_step[i];
      const T *g = c_base[i] + k0;   // uniform
      // M0 carries the LDS byte address; the compiler does not model this load, so the waits below are explicit
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2" : : "v"(c_voff[i]), "s"(off), "s"(g) : "memory");
    }
  };
  auto issue = [&](int buf, int k0) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) issue_one(buf, k0, i);
  };

  vacc acc[MB][NB];

  // ---- k loop.  A stage is one k-block of BK = 4*KV values, i.e. MB steps of NB*KV MFMAs (one A
  // fragment against the NB B fragments).  The loop body covers two stages so that every LDS
  // buffer and fragment slot is a compile-time choice.  Within a stage:
  //   * the LDS-direct loads of the next k-block go into the other buffer -- every wave finished reading that buffer
  //     before the previous barrier -- one at a time, spread over the steps of the stage;
  //   * every step fetches the next step's A fragment before issuing its own MFMAs;
  //   * the last step waits for this wave's loads (vmcnt), passes the barrier (after which the other
  //     buffer is complete) and fetches the first fragments of the next stage, so they arrive
  //     while the last MFMAs of this stage execute.
  static_assert(BK == 4 * KV, "one k-group per stage");
  const int npairs = a.ldin / (2 * BK);  // ldin is a multiple of 32, so the stage count is even
  const int lgs = lg ^ ((lr >> 1) & 3);  // 16-byte units of a row are stored XOR-swizzled: conflict-free fragment reads
  const T *Ar = As + lr * LROW + lgs * KV;
  const T *Br = Bs + (wave * 16 + lr) * LROW + lgs * KV;  // + nb * 64 rows
  vld bf[2][NB], af[2];

  issue(0, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) bf[0][nb] = *reinterpret_cast<const vld *>(Br + nb * 64 * LROW);
  af[0] = *reinterpret_cast<const vld *>(Ar);

  // The first pair of stages is a copy of the loop body whose first MFMA per accumulator takes a literal zero as its C
  // operand: no vector-ALU instructions to clear the accumulators (those of a starting workgroup would take issue
  // cycles from the MFMAs of the workgroup it shares the CU with).
  const int k_last = a.ldin - BK;
  constexpr bool kLoadMid = MB > 9;
  auto stage_pair = [&](int kp, auto first_tag) {
    constexpr bool kFirst = decltype(first_tag)::value;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      // stage `half` reads LDS buffer `half`; the next k-block goes straight to the other buffer, which every wave
      // finished reading before the previous barrier (the very last stage re-fetches its own block, unused)
      const int k_next = (2 * kp + half + 1) * BK < k_last ? (2 * kp + half + 1) * BK : k_last;
      const T *Ac = Ar + half * TL::A_STAGE;
      const T *An = Ar + (half ^ 1) * TL::A_STAGE;
      const T *Bn = Br + (half ^ 1) * TL::B_STAGE;
#pragma unroll
      for (int st = 0; st < MB; ++st) {
        const int s = half * MB + st;  // fragment slot parity runs across both stages
        if constexpr (!kLoadMid) {
#pragma unroll
          for (int i = 0; i < NCH; ++i)
            if (st == 1 + i * (MB - 1) / NCH) issue_one(half ^ 1, k_next, i);
        }
        if (st + 1 < MB) {
          af[(s + 1) & 1] = *reinterpret_cast<const vld *>(Ac + (st + 1) * 16 * LROW);
        } else {
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's share of the next stage has landed
          __syncthreads();
          af[(s + 1) & 1] = *reinterpret_cast<const vld *>(An);
#pragma unroll
          for (int nb = 0; nb < NB; ++nb) bf[half ^ 1][nb] = *reinterpret_cast<const vld *>(Bn + nb * 64 * LROW);
        }
        __builtin_amdgcn_sched_barrier(0);  // keep the fetches ahead of this step's MFMAs
#pragma unroll
        for (int j = 0; j < KV; ++j) {
          if (kLoadMid && j == KV / 2) {
            // this wave's loads of the next k-block, one at a time, spread over the steps of the stage instead of all at
            // its top (bursts of load instructions from every wave cost 1.2 %).  Tall tiles issue them in the middle of
            // a step's MFMA group, short ones (MB <= 9, four workgroups per CU) at the start of a step: measured, each
            // 0.3 - 4 % better than the other position on its tile heights.
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NCH; ++i)
              if (st == i * (MB - 1) / NCH) issue_one(half ^ 1, k_next, i);
            __builtin_amdgcn_sched_barrier(0);
          }
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
            acc[st][nb] = mfma16(af[s & 1][j], bf[half][nb][j], (kFirst && half == 0 && j == 0) ? vacc{0, 0, 0, 0} : acc[st][nb]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  // Tall tiles run the k loop at raised wave priority: where a SIMD has to choose between this wave's next MFMA (or
  // fragment read) and an instruction of a neighbour's prologue or epilogue, the MFMA stream goes first (MB = 13: +0.9 %,
  // any level above 0).  With four short workgroups per CU the same setting costs 3 % (MB = 9), so they keep level 0.
  if constexpr (MB > 9) __builtin_amdgcn_s_setprio(1);
  stage_pair(0, std::true_type{});
  for (int kp = 1; kp < npairs; ++kp) stage_pair(kp, std::false_type{});
  // Each wave's last real fragment read and its last (surplus) loads completed before it entered the final barrier
  // above, so the stages can be reused for the C tile right away (the fragments fetched after that barrier are unused).

  // ---- epilogue, one chunk of CCOLS output columns at a time (fp32: chunk c is the column block acc[.][c], wave w
  // holds its columns w*16 .. +15; fp64: chunk c is the 16 columns each of the waves 2c and 2c+1): stage that chunk of
  // the accumulators through LDS, then apply the collapsed jet rule with one thread per (point, feature) pair, walking
  // the point's rows in order.  With fp64 only the lower half of a wavefront has a column.
  if constexpr (MB > 9) __builtin_amdgcn_s_setprio(0);
  const int rho = a.rho;
  const int j = tid & 63;
  constexpr int CCOLS = TL::CCOLS;
  static_assert(BN / CCOLS == 2, "two chunks per tile");
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    if (nb > 0) __syncthreads();  // the previous chunk has been consumed
    if constexpr (NB == 2) {
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int v = 0; v < 4; ++v)
          Cs[(mb * 16 + Vec<T>::out_row(lg, v)) * CROW + wave * 16 + lr] = acc[mb][nb][v];
    } else {
      if ((wave_u >> 1) == nb) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int v = 0; v < 4; ++v)
            Cs[(mb * 16 + Vec<T>::out_row(lg, v)) * CROW + (wave_u & 1) * 16 + lr] = acc[mb][0][v];
      }
    }
    __syncthreads();

    const long jg = (long)col_tile * BN + nb * CCOLS + j;
    const bool col_ok = j < CCOLS && jg < a.ldout;
    const T bias = col_ok ? a.bias[jg] : T(0);
    const long ostep = a.ldout;
    if constexpr (WPP == 1) {  // a wavefront per point
      if (col_ok) {
        for (int p = wave_u; p < p_valid; p += kThreads / 64) {
          const T *c = Cs + p * rho * CROW + j;
          const long n = p0 + p;
          const long jg0 = (long)col_tile * BN + nb * CCOLS;  // the wavefront's first column: n, jg0 are wavefront-uniform
          const unsigned voff = (unsigned)(j * sizeof(T));
          T *o = a.Hout + (n * a.out_rows) * a.ldout + jg0;
          if constexpr (MODE == kReverse) {
            jet_rule_bwd<T>(c, CROW, a.Zsaved + (n * rho) * a.ldout + jg0, a.ldout, o, ostep, voff, a);
          } else {
            if constexpr (MODE == kTape) save_preactivations<T>(c, CROW, bias, a.Zout + (n * rho) * a.ldout + jg0, a.ldout, voff, rho);
            jet_rule<T, PlainRows<T>, 1, MODE == kStandard>(c, CROW, bias, PlainRows<T>{o, ostep, voff}, a);
          }
        }
      }
    } else {
      // tiles of one or two points: the point's directions are shared out over 4 or 2 wavefronts (every thread
      // takes part: the rule holds a barrier)
      const int p = WPP == 2 ? (wave_u >> 1) : 0;
      const int sub = WPP == 2 ? (wave_u & 1) : wave_u;
      const bool active = col_ok && p < p_valid;
      const T *c = Cs + p * rho * CROW + j;
      const long n = p0 + p;
      const long jg0 = (long)col_tile * BN + nb * CCOLS;
      const PlainRows<T> out{a.Hout + (n * a.out_rows) * a.ldout + jg0, ostep, (unsigned)(j * sizeof(T))};
      T *red = reinterpret_cast<T *>(lds_raw + TL::kRedOffset) + p * 2 * 64 + j;  // p > 0 only when two wavefronts share a point
      if constexpr (MODE == kTape) {
        if (active && sub == 0)
          save_preactivations<T>(c, CROW, bias, a.Zout + (n * rho) * a.ldout + jg0, a.ldout, (unsigned)(j * sizeof(T)), rho);
      }
      jet_rule<T, PlainRows<T>, WPP, false>(c, CROW, bias, out, a, active, sub, red);
    }
  }
}

template <typename T, int MB, int WPP, int MODE> static hipError_t launch_kernel(const LayerArgs<T> &a, hipStream_t s) {
  using TL = Tile<T, MB>;
  static LdsLimitOnce lds_limit;
  const size_t lds = TL::kRedOffset + (WPP > 1 ? TL::kRedBytes : 0);
  hipError_t e = lds_limit.ensure(reinterpret_cast<const void *>(&layer_kernel<T, MB, WPP, MODE>), lds);
  if (e != hipSuccess) return e;
  const long n_tiles = a.n_row_tiles * a.n_col_tiles;
  const long grid = (n_tiles + kXcds - 1) / kXcds * kXcds;
  if (grid <= 0 || grid > 0x7fffffffL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((layer_kernel<T, MB, WPP, MODE>), dim3((unsigned)grid), dim3(kThreads), lds, s, a);
  return hipGetLastError();
}

template <typename T, int MB, int WPP> static hipError_t launch_wpp(const LayerArgs<T> &a, hipStream_t s) {
  // the modes exclude one another: the reverse pass and the un-collapsed layout record no tape
  if ((a.bwd != 0) + (a.standard != 0) + (a.Zout != nullptr) > 1) return hipErrorInvalidValue;
  if (a.Zout != nullptr) return launch_kernel<T, MB, WPP, kTape>(a, s);
  if constexpr (WPP == 1) {  // wavefronts share points only in the collapsed forward passes
    if (a.bwd) return launch_kernel<T, MB, WPP, kReverse>(a, s);
    if (a.standard) return launch_kernel<T, MB, WPP, kStandard>(a, s);
  } else {
    if (a.bwd || a.standard) return hipErrorInvalidValue;
  }
  return launch_kernel<T, MB, WPP, kPlain>(a, s);
}

// wpp wavefronts share a point in the rule (tiles of 1 or 2 points; forward, collapsed mode only)
template <typename T, int MB> static hipError_t launch_one(const LayerArgs<T> &a, hipStream_t s) {
  if (a.wpp == 1) return launch_wpp<T, MB, 1>(a, s);
  if (a.bwd || a.standard || a.P * a.wpp != 4) return hipErrorInvalidValue;
  return a.wpp == 2 ? launch_wpp<T, MB, 2>(a, s) : launch_wpp<T, MB, 4>(a, s);
}

bool row_blocks_supported(int MB) {
  return MB == 4 || MB == 8 || MB == 9 || MB == 12 || MB == 13 || MB == 16;
}

template <typename T> hipError_t launch_layer(const LayerArgs<T> &a, int MB, hipStream_t s) {
  switch (MB) {
    case 4: return launch_one<T, 4>(a, s);
    case 8: return launch_one<T, 8>(a, s);
    case 9: return launch_one<T, 9>(a, s);
    case 12: return launch_one<T, 12>(a, s);
    case 13: return launch_one<T, 13>(a, s);
    case 16: return launch_one<T, 16>(a, s);
    default: return hipErrorInvalidValue;
  }
}

template hipError_t launch_layer<float>(const LayerArgs<float> &, int, hipStream_t);
template hipError_t launch_layer<double>(const LayerArgs<double> &, int, hipStream_t);

}  // namespace ctm
