// Plain-bf16 stacked GEMM with 256-column tiles (the operation, the MFMA use, the stage layout and the LDS-direct loads are
// those of the plain variant in ctm_layer_bf16.hip).
#include "ctm_internal.h"
#include "ctm_rule.h"

namespace ctm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreadsB = 256;
constexpr int kXcdsB = 8;

// The 16 x MB rows x 128 columns tile of that file is bound by the path that brings operands to LDS, not by the matrix pipe
// (measured on the 768-wide benchmark layers: the unit that returns loaded data to LDS busy 86-88 % of the cycles, the
// matrix pipe a third of them).  This variant halves the weight bytes and cuts the LDS fragment bytes per MFMA:
//   * 4 wavefronts side by side own 16 * MB rows x 256 columns; each computes ALL MB row blocks x 4 column blocks
//     (16 * MB accumulator registers: MB <= 13), so an A fragment feeds four MFMAs and no row block is padded;
//   * two workgroups per compute unit (59 KiB of stages / 55 KiB of staged C each): one's epilogue runs under the
//     other's main loop, which is bound by loads and leaves the vector ALU and most LDS cycles free;
//   * the MFMA operands are swapped (D^T = B A^T), so a lane holds four consecutive FEATURES of one coefficient row and
//     stages them with one 16-byte LDS store (only one wavefront owns the 64 columns of a chunk, and it stages alone).
// Same LDS-direct loads, stage layout, swizzle and epilogue rule as that plain variant.
template <int MB> struct TileT {
  static constexpr int BM = 16 * MB, BN = 256, BK = 32, PITCH = BK;
  static constexpr int A_PLANE = BM * PITCH, B_PLANE = BN * PITCH, STAGE = A_PLANE + B_PLANE;   // bf16 elements
  static constexpr int CROW = 64 + 4;    // floats; measured: the 16-byte staging stores are free of bank conflicts with this pitch (not with 72 or 80)
  static constexpr size_t kStageBytes = 2 * (size_t)STAGE * 2;
  static constexpr size_t kCBytes = (size_t)BM * CROW * 4;
  static constexpr size_t kRedOffset = ((kStageBytes > kCBytes ? kStageBytes : kCBytes) + 15) / 16 * 16;
  static constexpr size_t kRedBytes = 4 * 64 * sizeof(float);
  static constexpr size_t kLdsBytes = kRedOffset + kRedBytes;
  static_assert(MB <= 13, "16 * MB accumulator registers per lane");
  static_assert(2 * kLdsBytes <= 160 * 1024, "two workgroups per CU");
};

template <int MB, int WPP>
__global__ __launch_bounds__(kThreadsB) __attribute__((amdgpu_waves_per_eu(2, 2)))
void layer_kernel_bf16_t256(const LayerArgs<float> a) {
  using TL = TileT<MB>;
  constexpr int BN = TL::BN, BK = TL::BK, PITCH = TL::PITCH, CROW = TL::CROW;

  extern __shared__ __align__(16) unsigned char lds_raw[];
  __bf16 *lds = reinterpret_cast<__bf16 *>(lds_raw);
  float *Cs = reinterpret_cast<float *>(lds_raw);   // reuses the stages after the k loop

  const unsigned n_tiles = (unsigned)(a.n_row_tiles * a.n_col_tiles);   // below 2^31 (checked at launch)
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

  const long p0 = row_tile * a.P;
  const int p_valid = (int)((a.n_points - p0) < a.P ? (a.n_points - p0) : a.P);
  const int rows_valid = p_valid * a.rho;   // <= 16 * MB (checked at launch)
  const __bf16 *Ag = reinterpret_cast<const __bf16 *>(a.Hin) + p0 * a.rho * (long)a.ldin;
  const __bf16 *Bg = reinterpret_cast<const __bf16 *>(a.Whi) + (long)col_tile * BN * a.ldin;

  // LDS-direct loads as in the 128-column plain variant: chunks of 16 rows x 64 bytes, 0 .. MB-1 the A tile, then 16 of the B tile;
  // wave w takes chunks w, w+4, ...; address = uniform tile base + per-lane 32-bit byte offset
  constexpr int kChunks = MB + BN / 16;
  constexpr int NCH = (kChunks + 3) / 4;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  unsigned c_voff[NCH], c_off[NCH];
  const __bf16 *c_base[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = wave_u + 4 * i;
    const int rr = lane >> 2;
    const int uu = (lane & 3) ^ ((rr >> 1) & 3);
    if (c < MB) {
      const int row = c * 16 + rr;
      const int grow = row < rows_valid ? row : rows_valid - 1;
      c_voff[i] = (unsigned)(((long)grow * a.ldin + uu * 8) * 2);
      c_base[i] = Ag;
      c_off[i] = (unsigned)(c * 16 * PITCH * 2);
    } else {
      const int cb = c < kChunks ? c - MB : 0;
      c_voff[i] = (unsigned)(((long)(cb * 16 + rr) * a.ldin + uu * 8) * 2);
      c_base[i] = Bg;
      c_off[i] = (unsigned)((TL::A_PLANE + cb * 16 * PITCH) * 2);
    }
  }
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)lds_raw;
  auto issue = [&](int stage, int k0) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      if (wave_u + 4 * i < kChunks) {
        const unsigned off = lds_base + c_off[i] + (unsigned)(stage * TL::STAGE * 2);
        const __bf16 *g = c_base[i] + k0;   // uniform
        // M0 carries the LDS byte address; the compiler does not model this load, so the waits are explicit
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2" : : "v"(c_voff[i]), "s"(off), "s"(g) : "memory");
      }
    }
  };

  f32x4 acc[MB][4];
#pragma unroll
  for (int m = 0; m < MB; ++m)
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) acc[m][nb] = f32x4{0, 0, 0, 0};

  const int nk = a.ldin / BK;
  issue(0, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  const int lgs = lg ^ ((lr >> 1) & 3);   // swizzled unit (rows lr and 16 m + lr share bits 1..2)

  for (int kt = 0; kt < nk; ++kt) {
    const int stage = kt & 1;
    const int k_next = (kt + 1 < nk) ? (kt + 1) * BK : kt * BK;   // the last stage re-fetches itself (unused)
    issue(stage ^ 1, k_next);   // every wave finished reading that stage before the previous barrier
    const __bf16 *S = lds + stage * TL::STAGE;
    const __bf16 *Ah = S + lr * PITCH + lgs * 8;
    const __bf16 *Bh = S + TL::A_PLANE + (wave * 64 + lr) * PITCH + lgs * 8;
    bf16x8 bh[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb) bh[nb] = *reinterpret_cast<const bf16x8 *>(Bh + nb * 16 * PITCH);
    bf16x8 ah[2];
    ah[0] = *reinterpret_cast<const bf16x8 *>(Ah);
#pragma unroll
    for (int m = 0; m < MB; ++m) {
      if (m + 1 < MB) ah[(m + 1) & 1] = *reinterpret_cast<const bf16x8 *>(Ah + (m + 1) * 16 * PITCH);
      __builtin_amdgcn_sched_barrier(0);
      // operands swapped: the lane receives features 4 lg .. 4 lg + 3 of column block nb for coefficient row 16 m + lr
#pragma unroll
      for (int nb = 0; nb < 4; ++nb) acc[m][nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bh[nb], ah[m & 1], acc[m][nb], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's share of the next stage has landed
    __syncthreads();
  }

  // ---- epilogue: 64 output columns at a time; chunk c holds the columns of wave c, which stages them alone
  const int rho = a.rho;
  const int j = tid & 63;
  for (int chunk = 0; chunk < 4; ++chunk) {
    if (chunk > 0) __syncthreads();
    if (wave_u == chunk) {
#pragma unroll
      for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) *reinterpret_cast<f32x4 *>(Cs + (m * 16 + lr) * CROW + nb * 16 + lg * 4) = acc[m][nb];
    }
    __syncthreads();
    const long jg = (long)col_tile * BN + chunk * 64 + j;
    const bool col_ok = jg < a.ldout;
    const float bias = col_ok ? a.bias[jg] : 0.f;
    auto rule = [&](const float *c, long n, bool active, int sub, float *red) {
      const long o_off = (n * a.out_rows) * a.ldout + (long)col_tile * BN + chunk * 64;
      if (a.out_bf16)
        jet_rule<float, Bf16Rows, WPP, false>(c, CROW, bias, Bf16Rows{reinterpret_cast<__bf16 *>(a.Hout) + o_off, a.ldout, (unsigned)(j * 2)}, a, active, sub, red);
      else
        jet_rule<float, StreamRows<float>, WPP, false>(c, CROW, bias, StreamRows<float>{{a.Hout + o_off, a.ldout, (unsigned)(j * 4)}}, a, active, sub, red);
    };
    if constexpr (WPP == 1) {  // a wavefront per point
      if (!a.last) {
        // every row of every point goes out: the rule overwrites the chunk in place, and the finished chunk leaves with
        // 16-byte stores (as in the 128-column kernel)
        if (col_ok)
          for (int p = wave_u; p < p_valid; p += kThreadsB / 64)
            jet_rule<float, LdsRows<float>, 1, false>(Cs + p * rho * CROW + j, CROW, bias, LdsRows<float>{Cs + p * rho * CROW, CROW, (unsigned)(j * 4)}, a);
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

template <int MB, int WPP> static hipError_t launch_t256(const LayerArgs<float> &a, hipStream_t s) {
  using TL = TileT<MB>;
  static LdsLimitOnce lds_limit;
  const size_t lds = TL::kRedOffset + (WPP > 1 ? TL::kRedBytes : 0);
  hipError_t e = lds_limit.ensure(reinterpret_cast<const void *>(&layer_kernel_bf16_t256<MB, WPP>), lds);
  if (e != hipSuccess) return e;
  const long n_tiles = a.n_row_tiles * a.n_col_tiles;
  const long grid = (n_tiles + kXcdsB - 1) / kXcdsB * kXcdsB;
  if (grid <= 0 || grid > 0x7fffffffL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((layer_kernel_bf16_t256<MB, WPP>), dim3((unsigned)grid), dim3(kThreadsB), lds, s, a);
  return hipGetLastError();
}

// Built: tiles of 9, 12 and 13 row blocks with a wavefront per point, and 13 row blocks with two wavefronts per point.
bool bf16_t256_supported(int MB, int wpp) { return (wpp == 1 && (MB == 9 || MB == 12 || MB == 13)) || (wpp == 2 && MB == 13); }

hipError_t launch_layer_bf16_t256(const LayerArgs<float> &a, int MB, hipStream_t s) {
  // the shapes the kernel assumes, checked before anything is launched
  if (!bf16_t256_supported(MB, a.wpp) || a.bwd || a.standard || a.Zout != nullptr || a.Whi == nullptr) return hipErrorInvalidValue;
  if (a.ldin % 32 != 0 || a.P < 1 || (long)a.P * a.rho > 16L * MB || (a.wpp > 1 && a.P * a.wpp != 4)) return hipErrorInvalidValue;
  if (a.n_row_tiles != (a.n_points + a.P - 1) / a.P || (long)a.n_col_tiles * 256 < a.ldout) return hipErrorInvalidValue;
  if (a.wpp == 2) return launch_t256<13, 2>(a, s);
  switch (MB) {
    case 9: return launch_t256<9, 1>(a, s);
    case 12: return launch_t256<12, 1>(a, s);
    case 13: return launch_t256<13, 1>(a, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace ctm
