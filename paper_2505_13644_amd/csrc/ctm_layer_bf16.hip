// Stacked GEMM of one MLP layer on the bf16 matrix cores, fp32 storage and fp32 accumulation:
// the reduced-precision variants of layer_kernel (same tile of whole points, same epilogue rule).
//
//   NSPLIT = 3  "split bf16": every fp32 operand x is written as hi + lo with hi = bf16(x),
//               lo = bf16(x - hi); a*b is taken as a_hi*b_hi + a_hi*b_lo + a_lo*b_hi (the lo*lo
//               term, relative size 2^-16, is dropped) -- three v_mfma_f32_16x16x32_bf16 per block pair.
//   NSPLIT = 1  plain bf16 inputs: a_hi*b_hi only.
//
// Split variant: the coefficient block stays fp32 in HBM and the A tile is split while it is copied to LDS
// (measured faster than storing hi / lo planes, whose 2-byte stores double the epilogue's store count).
// Plain variant: between the layers the block lives in HBM as ONE bf16 plane [rows][ld] (half the traffic):
// every producer (the first-layer / seed kernels and this kernel's epilogue) rounds a value once, when it is
// written, and the GEMM copies its A tile to LDS as it is.  The last hidden layer's output rows are fp32 in
// both variants (they feed the final kernel).  The weights are split once at handle creation
// (Whi / Wlo, [rows_pad][ld] bf16).
//
// MFMA use: v_mfma_f32_16x16x32_bf16.  Lane l supplies 8 consecutive k values of A row l%16 and of
// B column l%16 (k = 8*(l/16) .. +7, the same assignment for both) and receives D rows
// 4*(l/16) .. +3 of column l%16.  Waves are arranged 2 x 2: each owns ceil(MB/2) row blocks and
// 4 column blocks, which keeps the LDS traffic per MFMA low enough for the 16-cycle instruction.
#include "ctm_internal.h"
#include "ctm_rule.h"

namespace ctm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreadsB = 256;
constexpr int kXcdsB = 8;

template <int MB, int NSPLIT> struct TileB {
  static constexpr int MBH = (MB + 1) / 2;        // row blocks per wave
  static constexpr int AROWS = 2 * MBH * 16;      // LDS rows of the A planes; rows >= 16*MB are never written
  static constexpr int BM = 16 * MB;
  static constexpr int BN = 128, BK = 32;
  // bf16 elements per LDS row: 64 B, unpadded; the four 16-byte units of a row are XOR-swizzled with bits 1..2 of the row
  // (conflict-free fragment reads, see layer_kernel).  The plain variant's rows arrive by LDS-direct loads (16 rows = 1 KiB
  // per wave instruction), the split variant writes them from registers; with its former 80-byte rows every fragment read
  // took twice the LDS cycles (benchmark layers: 1.77 -> 1.73 ms).
  static constexpr int PITCH = BK;
  static constexpr int PLANES = NSPLIT == 3 ? 2 : 1;
  static constexpr int A_PLANE = AROWS * PITCH;
  static constexpr int B_PLANE = BN * PITCH;
  static constexpr int STAGE = PLANES * (A_PLANE + B_PLANE);   // bf16 elements
  static constexpr int UPR = BK / 8;              // 8-element units per row (= 4)
  static constexpr int A_LD = (BM * UPR + kThreadsB - 1) / kThreadsB;
  static constexpr int B_LD = (BN * UPR) / kThreadsB;          // per plane
  // Workgroups per CU the kernel is compiled for: the plain variant's registers (8 * MB accumulators + fragments) allow
  // three up to MB = 13; its staged C chunk then drops the bank-conflict pad at MB = 13, which is what lets the third fit
  static constexpr int kWgPerCu = (NSPLIT == 1 && MB <= 13) ? 3 : 2;
  static constexpr int CROW = 64 + ((kWgPerCu == 3 && 3 * (size_t)BM * 68 * 4 > 160 * 1024) ? 0 : 4);
  // The split variant keeps ONE stage of its A planes in LDS (they are split from fp32 registers; two barriers per k
  // step) so that two workgroups fit a CU and cover each other's barriers, conversions and load latency; its weight
  // planes are bf16 in memory already and come by LDS-direct loads into a double buffer of their own, one k step ahead.
  // The plain variant's stage is half as large and is double-buffered as a whole.
  static constexpr int NSTAGE = NSPLIT == 3 ? 1 : 2;
  static constexpr int B_BUF = PLANES * B_PLANE;   // split: one buffer of the weight planes [hi][lo]
  static constexpr size_t kStageBytes = NSPLIT == 3 ? ((size_t)PLANES * A_PLANE + 2 * (size_t)B_BUF) * 2 : NSTAGE * (size_t)STAGE * 2;
  static constexpr size_t kCBytes = (size_t)BM * CROW * 4;
  // behind them: the group sums that wavefronts sharing a point exchange (2 point slots x 4 groups x 64 columns)
  static constexpr size_t kRedOffset = ((kStageBytes > kCBytes ? kStageBytes : kCBytes) + 15) / 16 * 16;
  static constexpr size_t kRedBytes = 4 * 64 * sizeof(float);   // only allocated by the kernels that share points (WPP > 1)
  static constexpr size_t kLdsBytes = kRedOffset + kRedBytes;
  static_assert(kLdsBytes <= 160 * 1024, "tile does not fit the 160 KiB LDS of a CU");
};

__device__ __forceinline__ void split8(const f32x4 &x0, const f32x4 &x1, bf16x8 &hi, bf16x8 &lo) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const __bf16 h0 = (__bf16)x0[i], h1 = (__bf16)x1[i];
    hi[i] = h0;
    hi[4 + i] = h1;
    lo[i] = (__bf16)(x0[i] - (float)h0);
    lo[4 + i] = (__bf16)(x1[i] - (float)h1);
  }
}

template <int MB, int NSPLIT, int WPP>
__global__ __launch_bounds__(kThreadsB) __attribute__((amdgpu_waves_per_eu(TileB<MB, NSPLIT>::kWgPerCu, TileB<MB, NSPLIT>::kWgPerCu)))
void layer_kernel_bf16(const LayerArgs<float> a) {
  using TL = TileB<MB, NSPLIT>;
  constexpr int MBH = TL::MBH, BN = TL::BN, BK = TL::BK, PITCH = TL::PITCH, UPR = TL::UPR, CROW = TL::CROW;
  constexpr bool SPLIT = NSPLIT == 3;

  extern __shared__ __align__(16) unsigned char lds_raw[];
  __bf16 *lds = reinterpret_cast<__bf16 *>(lds_raw);
  float *Cs = reinterpret_cast<float *>(lds_raw);   // reuses the stages after the k loop

  const unsigned n_tiles = (unsigned)(a.n_row_tiles * a.n_col_tiles);   // below 2^31 (checked at launch): 32-bit index arithmetic
  const unsigned xcd = blockIdx.x % kXcdsB;
  const unsigned slot = blockIdx.x / kXcdsB;
  const unsigned base = n_tiles / kXcdsB, rem = n_tiles % kXcdsB;
  const unsigned mine = base + (xcd < rem ? 1 : 0);
  if (slot >= mine) return;
  const unsigned tile = xcd * base + (xcd < rem ? xcd : rem) + slot;
  const long row_tile = tile / (unsigned)a.n_col_tiles;
  const int col_tile = (int)(tile % (unsigned)a.n_col_tiles);

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 15, lg = lane >> 4;
  const int wr = wave >> 1, wc = wave & 1;   // wave grid: row half, column half

  const long p0 = row_tile * a.P;
  const int p_valid = (int)((a.n_points - p0) < a.P ? (a.n_points - p0) : a.P);
  const int rows_valid = p_valid * a.rho;
  const float *Af_g = a.Hin + p0 * a.rho * (long)a.ldin;                                            // split: fp32 rows
  const __bf16 *Ah_g = reinterpret_cast<const __bf16 *>(a.Hin) + p0 * a.rho * (long)a.ldin;        // plain: bf16 plane
  const __bf16 *Bhi = reinterpret_cast<const __bf16 *>(a.Whi) + (long)col_tile * BN * a.ldin;
  const __bf16 *Blo = reinterpret_cast<const __bf16 *>(a.Wlo) + (long)col_tile * BN * a.ldin;

  // global -> LDS copy slots: 8 consecutive k values each (split: 32 B of fp32; plain: 16 B of bf16; weights: 16 B per
  // plane); unconditional, clamped as in layer_kernel
  int a_off[TL::A_LD];
  long a_src[TL::A_LD];
#pragma unroll
  for (int i = 0; i < TL::A_LD; ++i) {
    int u = tid + i * kThreadsB;
    u = u < TL::BM * UPR ? u : TL::BM * UPR - 1;
    const int row = u / UPR, q = u % UPR;
    a_off[i] = row * PITCH + (q ^ ((row >> 1) & 3)) * 8;
    const int grow = row < rows_valid ? row : rows_valid - 1;
    a_src[i] = (long)grow * a.ldin + q * 8;
  }
  f32x4 ga[SPLIT ? TL::A_LD : 1][2];
  bf16x8 gah[SPLIT ? 1 : TL::A_LD];
  auto load_global = [&](int k0) {
#pragma unroll
    for (int i = 0; i < TL::A_LD; ++i) {
      if constexpr (SPLIT) {
        ga[i][0] = *reinterpret_cast<const f32x4 *>(Af_g + a_src[i] + k0);
        ga[i][1] = *reinterpret_cast<const f32x4 *>(Af_g + a_src[i] + k0 + 4);
      } else {
        gah[i] = *reinterpret_cast<const bf16x8 *>(Ah_g + a_src[i] + k0);
      }
    }
  };
  // split layout: [A hi][A lo] then two weight buffers [B hi][B lo]; the A planes are written here, from registers
  auto store_lds = [&]() {
    __bf16 *Ah = lds, *Al = lds + TL::A_PLANE;
#pragma unroll
    for (int i = 0; i < TL::A_LD; ++i) {
      if constexpr (SPLIT) {
        bf16x8 hi, lo;
        split8(ga[i][0], ga[i][1], hi, lo);
        *reinterpret_cast<bf16x8 *>(Ah + a_off[i]) = hi;
        *reinterpret_cast<bf16x8 *>(Al + a_off[i]) = lo;
      } else {
        *reinterpret_cast<bf16x8 *>(Ah + a_off[i]) = gah[i];
      }
    }
  };

  // Plain variant: both operands are bf16 in HBM, so a k-block goes straight to LDS by LDS-direct loads
  // (global_load_lds_dwordx4: lane l of a wave brings row l/4, 16-byte unit (l%4) ^ ((l/4 >> 1) & 3) of a 16-row chunk to
  // LDS address M0 + 16*l).  Chunks 0..MB-1 are the A tile, MB..MB+7 the B tile; wave w takes chunks w, w+4, ...
  constexpr int kChunks = MB + BN / 16;
  constexpr int NCH = (kChunks + 3) / 4;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const __bf16 *c_src[NCH];
  unsigned c_off[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = wave_u + 4 * i;
    const int rr = lane >> 2;
    const int uu = (lane & 3) ^ ((rr >> 1) & 3);
    if (c < MB) {
      const int row = c * 16 + rr;
      const int grow = row < rows_valid ? row : rows_valid - 1;
      c_src[i] = Ah_g + (long)grow * a.ldin + uu * 8;
      c_off[i] = (unsigned)(c * 16 * PITCH * 2);
    } else {
      const int cb = c < kChunks ? c - MB : 0;
      c_src[i] = Bhi + (long)(cb * 16 + rr) * a.ldin + uu * 8;
      c_off[i] = (unsigned)((TL::A_PLANE + cb * 16 * PITCH) * 2);
    }
  }
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)lds_raw;
  auto issue = [&](int stage, int k0) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      if (wave_u + 4 * i < kChunks) {
        const unsigned off = lds_base + c_off[i] + (unsigned)(stage * TL::STAGE * 2);
        const __bf16 *g = c_src[i] + k0;
        // M0 carries the LDS byte address; the compiler does not model this load, so the waits are explicit
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(g), "s"(off) : "memory");
      }
    }
  };

  // Split variant: the weight planes the same way into their own double buffer.  16 chunks of 16 rows (8 of the hi plane,
  // then 8 of the lo plane); wave w takes chunks w, w + 4, w + 8, w + 12.  Address = uniform plane base + per-lane offset.
  constexpr int kBChunks = 2 * BN / 16;
  auto issue_b = [&](int buf, int k0) {
    const int rr = lane >> 2;
    const unsigned voff = (unsigned)(((long)rr * a.ldin + ((lane & 3) ^ ((rr >> 1) & 3)) * 8) * 2);   // < 2^32: 16 rows of ldin
#pragma unroll
    for (int i = 0; i < kBChunks / 4; ++i) {
      const int c = wave_u + 4 * i;                 // uniform
      const int plane = c / (BN / 16), cb = c % (BN / 16);
      const __bf16 *g = (plane ? Blo : Bhi) + (long)cb * 16 * a.ldin + k0;
      const unsigned off = lds_base + (unsigned)((TL::PLANES * TL::A_PLANE + buf * TL::B_BUF + plane * TL::B_PLANE + cb * 16 * PITCH) * 2);
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2" : : "v"(voff), "s"(off), "s"(g) : "memory");
    }
  };

  f32x4 acc[MBH][4];
#pragma unroll
  for (int m = 0; m < MBH; ++m)
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) acc[m][nb] = f32x4{0, 0, 0, 0};

  const int nk = a.ldin / BK;
  if constexpr (SPLIT) {
    issue_b(0, 0);
    load_global(0);
    store_lds();
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  } else {
    issue(0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  __syncthreads();
  const int lgs = lg ^ ((lr >> 1) & 3);  // swizzled unit (rows lr and 16*m + lr share bits 1..2)

  for (int kt = 0; kt < nk; ++kt) {
    const int stage = TL::NSTAGE == 2 ? (kt & 1) : 0;
    const int k_next = (kt + 1 < nk) ? (kt + 1) * BK : kt * BK;   // last stage re-fetches itself (unused)
    if constexpr (SPLIT) {
      // weights of the next k step into the other weight buffer (every wave finished reading it before the previous
      // barrier), issued ahead of the fp32 loads so that the compiler's waits for those also cover these
      issue_b((kt & 1) ^ 1, k_next);
      load_global(k_next);
    } else {
      issue(stage ^ 1, k_next);   // every wave finished reading that stage before the previous barrier
    }

    const __bf16 *S = lds + stage * TL::STAGE;   // split: stage == 0, the single A stage
    const __bf16 *Ah = S + (wr * MBH * 16 + lr) * PITCH + lgs * 8;
    const __bf16 *Al = Ah + TL::A_PLANE;
    const __bf16 *Bh = (SPLIT ? lds + TL::PLANES * TL::A_PLANE + (kt & 1) * TL::B_BUF : S + TL::PLANES * TL::A_PLANE) + (wc * 64 + lr) * PITCH + lgs * 8;
    const __bf16 *Bl = Bh + TL::B_PLANE;
    bf16x8 bh[4], bl[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) {
      bh[nb] = *reinterpret_cast<const bf16x8 *>(Bh + nb * 16 * PITCH);
      if (SPLIT) bl[nb] = *reinterpret_cast<const bf16x8 *>(Bl + nb * 16 * PITCH);
    }
    bf16x8 ah[2], al[2];
    ah[0] = *reinterpret_cast<const bf16x8 *>(Ah);
    if (SPLIT) al[0] = *reinterpret_cast<const bf16x8 *>(Al);
#pragma unroll
    for (int m = 0; m < MBH; ++m) {
      if (m + 1 < MBH) {  // next row block's fragments, fetched ahead of this block's MFMAs
        ah[(m + 1) & 1] = *reinterpret_cast<const bf16x8 *>(Ah + (m + 1) * 16 * PITCH);
        if (SPLIT) al[(m + 1) & 1] = *reinterpret_cast<const bf16x8 *>(Al + (m + 1) * 16 * PITCH);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int nb = 0; nb < 4; ++nb) {
        acc[m][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah[m & 1], bh[nb], acc[m][nb], 0, 0, 0);
        if (SPLIT) {
          acc[m][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah[m & 1], bl[nb], acc[m][nb], 0, 0, 0);
          acc[m][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al[m & 1], bh[nb], acc[m][nb], 0, 0, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }

    if constexpr (SPLIT) {
      __syncthreads();        // every wave finished reading the A stage
      store_lds();
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's share of the next stage (split: of the next weights) has landed
    __syncthreads();
  }

  // ---- epilogue: 64 output columns at a time.  Chunk c holds the columns of the waves with wc == c.
  const int rho = a.rho;
  const int j = tid & 63;
  for (int chunk = 0; chunk < 2; ++chunk) {
    if (chunk > 0) __syncthreads();
    if (wc == chunk) {
#pragma unroll
      for (int m = 0; m < MBH; ++m) {
        const int mb = wr * MBH + m;
        if (mb < MB) {
#pragma unroll
          for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int v = 0; v < 4; ++v) Cs[(mb * 16 + lg * 4 + v) * CROW + nb * 16 + lr] = acc[m][nb][v];
        }
      }
    }
    __syncthreads();
    const long jg = (long)col_tile * BN + chunk * 64 + j;
    const bool col_ok = jg < a.ldout;
    const float bias = col_ok ? a.bias[jg] : 0.f;
    // n (the point) is wavefront-uniform: the output row addresses are scalar, the lane's column is a byte offset
    auto rule = [&](const float *c, long n, bool active, int sub, float *red) {
      const long o_off = (n * a.out_rows) * a.ldout + (long)col_tile * BN + chunk * 64;
      if (a.out_bf16)
        jet_rule<float, Bf16Rows, WPP>(c, CROW, bias, Bf16Rows{reinterpret_cast<__bf16 *>(a.Hout) + o_off, a.ldout, (unsigned)(j * 2)}, a, active, sub, red);
      else
        jet_rule<float, StreamRows<float>, WPP>(c, CROW, bias, StreamRows<float>{{a.Hout + o_off, a.ldout, (unsigned)(j * 4)}}, a, active, sub, red);
    };
    if constexpr (WPP == 1) {  // a wavefront per point
      if (!a.last) {
        // every row of every point goes out: the rule overwrites the chunk in place, and the finished chunk leaves with
        // 16-byte stores (a quarter / an eighth of the store instructions of one element per lane and row)
        if (col_ok)
          for (int p = wave_u; p < p_valid; p += kThreadsB / 64)
            jet_rule<float, LdsRows<float>, 1>(Cs + p * rho * CROW + j, CROW, bias, LdsRows<float>{Cs + p * rho * CROW, CROW, (unsigned)(j * 4)}, a);
        __syncthreads();
        const long jg0 = (long)col_tile * BN + chunk * 64;
        const long orow0 = p0 * rho;   // rows per point in the output block = rho (not the last hidden layer)
        if (a.out_bf16) {
          const int q = tid & 7;       // 8 lanes x 8 features per row
          if (jg0 + q * 8 < a.ldout)
            for (int r = tid >> 3; r < rows_valid; r += kThreadsB / 8) {
              const f32x4 x0 = *reinterpret_cast<const f32x4 *>(Cs + r * CROW + q * 8), x1 = *reinterpret_cast<const f32x4 *>(Cs + r * CROW + q * 8 + 4);
              bf16x8 v;
#pragma unroll
              for (int i = 0; i < 4; ++i) { v[i] = (__bf16)x0[i]; v[4 + i] = (__bf16)x1[i]; }
              __builtin_nontemporal_store(v, reinterpret_cast<bf16x8 *>(reinterpret_cast<__bf16 *>(a.Hout) + (orow0 + r) * a.ldout + jg0 + q * 8));
            }
        } else {
          const int q = tid & 15;      // 16 lanes x 4 features per row
          if (jg0 + q * 4 < a.ldout)
            for (int r = tid >> 4; r < rows_valid; r += kThreadsB / 16)
              __builtin_nontemporal_store(*reinterpret_cast<const f32x4 *>(Cs + r * CROW + q * 4), reinterpret_cast<f32x4 *>(a.Hout + (orow0 + r) * a.ldout + jg0 + q * 4));
        }
      } else if (col_ok) {
        for (int p = wave_u; p < p_valid; p += kThreadsB / 64)
          rule(Cs + p * rho * CROW + j, p0 + p, true, 0, nullptr);
      }
    } else {  // one or two points per tile: 4 or 2 wavefronts share a point's directions (see jet_rule)
      const int p = WPP == 2 ? (wave_u >> 1) : 0;
      const int sub = WPP == 2 ? (wave_u & 1) : wave_u;
      const bool active = col_ok && p < p_valid;
      float *red = reinterpret_cast<float *>(lds_raw + TL::kRedOffset) + p * 2 * 64 + j;
      rule(Cs + (long)p * rho * CROW + j, p0 + p, active, sub, red);
    }
  }
}

template <int MB, int NSPLIT, int WPP> static hipError_t launch_wpp_b(const LayerArgs<float> &a, hipStream_t s) {
  using TL = TileB<MB, NSPLIT>;
  static LdsLimitOnce lds_limit;
  hipError_t e = lds_limit.ensure(reinterpret_cast<const void *>(&layer_kernel_bf16<MB, NSPLIT, WPP>), TL::kRedOffset + (WPP > 1 ? TL::kRedBytes : 0));
  if (e != hipSuccess) return e;
  const long n_tiles = a.n_row_tiles * a.n_col_tiles;
  const long grid = (n_tiles + kXcdsB - 1) / kXcdsB * kXcdsB;
  if (grid <= 0 || grid > 0x7fffffffL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((layer_kernel_bf16<MB, NSPLIT, WPP>), dim3((unsigned)grid), dim3(kThreadsB), TL::kRedOffset + (WPP > 1 ? TL::kRedBytes : 0), s, a);
  return hipGetLastError();
}

template <int MB, int NSPLIT> static hipError_t launch_one_b(const LayerArgs<float> &a, hipStream_t s) {
  if (a.wpp == 1) return launch_wpp_b<MB, NSPLIT, 1>(a, s);
  if (a.bwd || a.standard || a.P * a.wpp != 4) return hipErrorInvalidValue;
  return a.wpp == 2 ? launch_wpp_b<MB, NSPLIT, 2>(a, s) : launch_wpp_b<MB, NSPLIT, 4>(a, s);
}

template <int NSPLIT> static hipError_t dispatch_b(const LayerArgs<float> &a, int MB, hipStream_t s) {
  switch (MB) {
    case 4: return launch_one_b<4, NSPLIT>(a, s);
    case 8: return launch_one_b<8, NSPLIT>(a, s);
    case 9: return launch_one_b<9, NSPLIT>(a, s);
    case 12: return launch_one_b<12, NSPLIT>(a, s);
    case 13: return launch_one_b<13, NSPLIT>(a, s);
    case 16: return launch_one_b<16, NSPLIT>(a, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_layer_bf16(const LayerArgs<float> &a, int MB, int nsplit, hipStream_t s) {
  return nsplit == 3 ? dispatch_b<3>(a, MB, s) : dispatch_b<1>(a, MB, s);
}

// ---- weights for the bf16 kernels: hi = bf16(w), lo = bf16(w - hi), zero-padded [rows_pad][ld]
__global__ void pack_bf16_kernel(const float *W, int d_out, int d_in, __bf16 *hi, __bf16 *lo, int rows_pad, int ld) {
  const long total = (long)rows_pad * ld;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const int k = (int)(i % ld);
    const int jrow = (int)(i / ld);
    const float w = (jrow < d_out && k < d_in) ? W[(long)jrow * d_in + k] : 0.f;
    const __bf16 h = (__bf16)w;
    hi[i] = h;
    lo[i] = (__bf16)(w - (float)h);
  }
}

hipError_t launch_pack_bf16(const float *W, int d_out, int d_in, void *hi, void *lo, int rows_pad, int ld, hipStream_t s) {
  const long total = (long)rows_pad * ld;
  long blocks = (total + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(pack_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, s, W, d_out, d_in,
                     reinterpret_cast<__bf16 *>(hi), reinterpret_cast<__bf16 *>(lo), rows_pad, ld);
  return hipGetLastError();
}

}  // namespace ctm
