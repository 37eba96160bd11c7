// Reverse pass of the collapsed propagation, orders 2 and 4 (gradients with respect to the weights):
// everything except the cotangent GEMM, which reuses layer_kernel with its reverse-rule epilogue.
//
// With L = sum_n gu_n u_n + gop_n op_n, u = w.h_0 + b, op = scale * w.h_2 at the last layer and, per hidden
// layer, Z = H_prev W^T (+ bias on the order-0 rows) followed by the rule (ctm_rule.h):
//   cotangents at the last hidden layer:  hb_0 = gu w,  hb_K = scale gop w, all other rows 0   -> bwd_last_kernel
//   dL/dw = sum_n gu_n h_0(n) + scale gop_n h_K(n),  dL/db_last = sum_n gu_n                  -> last_grads
//   (a network with C outputs has one (u, op) pair, one row of w and one bias per output; the cotangents sum over them)
//   per hidden layer:  dL/db = sum_n Zbar[order-0 row of n]                                    -> bias_grad
//                      dL/dW = Zbar^T H_prev   (a GEMM whose k index runs over all N*rho rows)  -> wgrad_kernel
//                      Hbar_prev = Zbar W, then the reverse rule                                -> layer_kernel (bwd)
// All reductions over points use fixed partitions and a fixed summation order (no atomics).
#include "ctm_internal.h"

#include <type_traits>
#include "ctm_rule.h"

namespace ctm {

// ---- cotangents of the last hidden layer's pre-activations ------------------------------------
template <typename T> __global__ void bwd_last_kernel(const BwdLastArgs<T> a) {
  const long total = a.N * a.ld;
  const int R = a.R, rho = a.rho;
  const long step = a.ld;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const int j = (int)(i % a.ld);
    const long n = i / a.ld;
    const T *zs = a.Z + (n * rho) * step + j;
    T *o = a.Zbar + (n * rho) * step + j;
    T hb0 = T(0), hbK = T(0);  // cotangents of h_0 and of the collapsed highest-order row; all others are zero
    for (int c = 0; c < a.C; ++c) {
      const T w = a.w[(long)c * a.ld + j];
      if (a.gu) hb0 += a.gu[n * a.C + c] * w;
      if (a.gop) hbK += (T)(a.scale * (double)a.gop[n * a.C + c]) * w;
    }
    T t, d1;
    act_eval<T>(a.act, zs[0], t, d1);
    const T d2 = act_d2<T>(a.act, t, d1), d3 = act_d3<T>(a.act, t, d1);
    if (a.order == 2) {
      // four directions per trip so that their loads are in flight together (the compiler may not move a load across
      // the store before it: it cannot tell that the two blocks do not overlap)
      const T w2 = T(2) * d2 * hbK;
      T sg[4] = {T(0), T(0), T(0), T(0)};
      int r = 1;
      for (; r + 3 <= R; r += 4) {
        T z1[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) z1[k] = zs[(r + k) * step];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          sg[k] += z1[k] * z1[k];
          o[(r + k) * step] = w2 * z1[k];
        }
      }
      for (int k = 0; r <= R; ++r, ++k) {
        const T z1 = zs[r * step];
        sg[k] += z1 * z1;
        o[r * step] = w2 * z1;
      }
      const T s = (sg[0] + sg[1]) + (sg[2] + sg[3]);
      o[(R + 1) * step] = d1 * hbK;
      o[0] = d1 * hb0 + d2 * hbK * zs[(R + 1) * step] + d3 * s * hbK;
    } else {  // the order-4 reverse rule (ctm_rule.h) with hb_1 = hb_2 = hb_3 = 0
      const T d4 = act_d4<T>(a.act, t, d1), d5 = act_d5<T>(a.act, t, d1);
      T s4 = T(0);
      for (int r = 0; r < R; ++r) {
        const T *zr = zs + (long)(1 + 3 * r) * step;
        T *orow = o + (long)(1 + 3 * r) * step;
        const T z1 = zr[0], z2 = zr[step], z3 = zr[2 * step];
        const T z1s = z1 * z1;
        orow[0] = T(4) * (d4 * z1s * z1 + T(3) * d3 * z1 * z2 + d2 * z3) * hbK;
        orow[step] = T(6) * (d3 * z1s + d2 * z2) * hbK;
        orow[2 * step] = T(4) * d2 * z1 * hbK;
        s4 += d5 * z1s * z1s + T(6) * d4 * z1s * z2 + T(4) * d3 * z1 * z3 + T(3) * d3 * z2 * z2;
      }
      o[(long)(3 * R + 1) * step] = d1 * hbK;
      o[0] = d1 * hb0 + hbK * (d2 * zs[(long)(3 * R + 1) * step] + s4);
    }
  }
}

template <typename T> hipError_t launch_bwd_last(const BwdLastArgs<T> &a, hipStream_t s) {
  long blocks = (a.N * a.ld + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(bwd_last_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}
template hipError_t launch_bwd_last<float>(const BwdLastArgs<float> &, hipStream_t);
template hipError_t launch_bwd_last<double>(const BwdLastArgs<double> &, hipStream_t);

// ---- column sums over the points, two stages with a fixed partition --------------------------------
constexpr int kSumChunks = 64;

// stage 1: partial[c][j] = sum over the rows n of chunk c of
//   weighted == 0:  X[n*row_stride + j]
//   weighted == 1:  ca[n*cs] * X[n*row_stride + j] + sb * cb[n*cs] * X[n*row_stride + second + j]   (a NULL vector counts as zeros)
template <typename T>
__global__ void colsum_stage1(const T *X, long row_stride, long second, int weighted, const T *ca, const T *cb, long cs, double sb,
                              long N, int ld, T *partial) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const int c = blockIdx.y;
  if (j >= ld) return;
  const long per = (N + kSumChunks - 1) / kSumChunks;
  const long n0 = c * per, n1 = (n0 + per < N) ? n0 + per : N;
  T acc = T(0);
  for (long n = n0; n < n1; ++n) {
    const T *row = X + n * row_stride + j;
    T v = row[0];
    if (weighted) v = (ca ? ca[n * cs] : T(0)) * row[0] + (T)(sb * (double)(cb ? cb[n * cs] : T(0))) * row[second];
    acc += v;
  }
  partial[(long)c * ld + j] = acc;
}

// stage 2: out[j] = sum_c partial[c][j], j < d.  Block 0 also sums vec[n*vs], n < N, into vec_sum[0] if asked.
// accumulate != 0: the sums are added to what out / vec_sum hold (several reverse passes into one gradient).
template <typename T>
__global__ void colsum_stage2(const T *partial, int ld, int d, T *out, const T *vec, long vs, long N, T *vec_sum, int accumulate) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < d) {
    T acc = T(0);
    for (int c = 0; c < kSumChunks; ++c) acc += partial[(long)c * ld + j];
    out[j] = accumulate ? out[j] + acc : acc;
  }
  if (vec_sum != nullptr && blockIdx.x == 0) {
    // one wavefront sums the vector in a fixed order
    __shared__ T red[256];
    T acc = T(0);
    if (vec != nullptr)
      for (long n = threadIdx.x; n < N; n += blockDim.x) acc += vec[n * vs];
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off >= 1; off >>= 1) {
      if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
      __syncthreads();
    }
    if (threadIdx.x == 0) vec_sum[0] = accumulate ? vec_sum[0] + red[0] : red[0];
  }
}

template <typename T>
hipError_t launch_last_grads(const T *pair, const T *gu, const T *gop, double scale, long N, int ld, int d, int C, T *gw, T *gbias,
                             T *scratch, hipStream_t s, int accumulate) {
  // per output: the order-0 row weighted by gu[:, c] plus the collapsed row weighted by scale * gop[:, c]
  for (int c = 0; c < C; ++c) {
    const T *guc = gu ? gu + c : nullptr, *gopc = gop ? gop + c : nullptr;
    hipLaunchKernelGGL(colsum_stage1<T>, dim3((ld + 255) / 256, kSumChunks), dim3(256), 0, s, pair, (long)2 * ld, (long)ld, 1, guc,
                       gopc, (long)C, scale, N, ld, scratch);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(colsum_stage2<T>, dim3((ld + 255) / 256), dim3(256), 0, s, scratch, ld, d, gw + (long)c * d, guc, (long)C, N,
                       gbias + c, accumulate);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}
template hipError_t launch_last_grads<float>(const float *, const float *, const float *, double, long, int, int, int, float *,
                                             float *, float *, hipStream_t, int);
template hipError_t launch_last_grads<double>(const double *, const double *, const double *, double, long, int, int, int, double *,
                                              double *, double *, hipStream_t, int);

template <typename T>
hipError_t launch_bias_grad(const T *Zbar, long N, int rho, int ld, int d, T *gb, T *scratch, hipStream_t s, int accumulate) {
  hipLaunchKernelGGL(colsum_stage1<T>, dim3((ld + 255) / 256, kSumChunks), dim3(256), 0, s, Zbar, (long)rho * ld, (long)0, 0,
                     (const T *)nullptr, (const T *)nullptr, (long)1, 0.0, N, ld, scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(colsum_stage2<T>, dim3((ld + 255) / 256), dim3(256), 0, s, scratch, ld, d, gb, (const T *)nullptr, (long)1, (long)0,
                     (T *)nullptr, accumulate);
  return hipGetLastError();
}
template hipError_t launch_bias_grad<float>(const float *, long, int, int, int, float *, float *, hipStream_t, int);
template hipError_t launch_bias_grad<double>(const double *, long, int, int, int, double *, double *, hipStream_t, int);

// ---- weight gradient: C[i][j] = sum_m Zbar[m][i] H[m][j] ---------------------------------------------
// Both operands are read as stored (k = row index m, feature index contiguous), so an LDS stage is
// [16 k][128 features] per operand and a lane picks single elements: A[i = l%16][k = l/16] = stage[k][i].
// A workgroup owns a 128 x 128 output tile over one range of rows; waves are 2 x 2, 4 x 4 MFMA blocks each.
typedef float wf32x4 __attribute__((ext_vector_type(4)));
typedef double wf64x4 __attribute__((ext_vector_type(4)));
template <typename T> struct WVec;
template <> struct WVec<float> {
  using acc = wf32x4;
  using ld4 = wf32x4;
  static __device__ __forceinline__ int out_row(int g, int v) { return g * 4 + v; }
  static __device__ __forceinline__ acc mfma(float a, float b, acc c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }
};
template <> struct WVec<double> {
  using acc = wf64x4;
  using ld4 = wf64x4;
  static __device__ __forceinline__ int out_row(int g, int v) { return v * 4 + g; }
  static __device__ __forceinline__ acc mfma(double a, double b, acc c) { return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0); }
};

constexpr int kWgTile = 128;
constexpr int kWgK = 16;               // rows per stage
constexpr int kWgPitch = kWgTile + 16; // LDS row pitch in elements: the four k rows a wave reads land in distinct banks
constexpr int kWgTargetBlocks = 1024;  // about two rounds of resident workgroups

struct WgradPlan {
  int ti, tj, ksplit, tile_i, tile_j;
  long rows_per;
};
// tile_i x tile_j outputs per workgroup: 128 x 128, or 256 x 64 (fp32 kernel, inputs of at most 64 features: the first
// layer of a low-dimensional problem would fill half of a 128-column tile or less)
static WgradPlan wgrad_plan(long M, int d_out, int d_in, bool narrow) {
  WgradPlan p;
  p.tile_i = narrow ? 2 * kWgTile : kWgTile;
  p.tile_j = narrow ? kWgTile / 2 : kWgTile;
  p.ti = (d_out + p.tile_i - 1) / p.tile_i;
  p.tj = (d_in + p.tile_j - 1) / p.tile_j;
  long ks = kWgTargetBlocks / ((long)p.ti * p.tj);
  const long max_ks = (M + 8 * kWgK - 1) / (8 * kWgK);  // at least eight stages per block
  if (ks > max_ks) ks = max_ks;
  if (ks > 1024) ks = 1024;
  if (ks < 1) ks = 1;
  p.rows_per = ((M + ks - 1) / ks + kWgK - 1) / kWgK * kWgK;
  p.ksplit = (int)((M + p.rows_per - 1) / p.rows_per);
  return p;
}
static bool wgrad_narrow(int d_in, bool fp32) { return fp32 && d_in <= kWgTile / 2; }
size_t wgrad_partial_elems(long M, int d_out, int d_in) {
  // the caller's buffer serves either precision: the larger of the two plans
  size_t need = 0;
  for (int fp32 = 0; fp32 < 2; ++fp32) {
    const WgradPlan p = wgrad_plan(M, d_out, d_in, wgrad_narrow(d_in, fp32 != 0));
    const size_t n = (size_t)p.ksplit * p.ti * p.tile_i * p.tj * p.tile_j;
    if (n > need) need = n;
  }
  return need;
}

template <typename T>
__global__ __launch_bounds__(256) void wgrad_kernel(const T *Zb, int ld_out, const T *H, int ld_in, long M, long rows_per, int tj,
                                                    T *partials) {
  using V = WVec<T>;
  using vacc = typename V::acc;
  using v4 = typename V::ld4;
  extern __shared__ __align__(16) unsigned char wg_lds[];
  T(*As)[kWgK][kWgPitch] = reinterpret_cast<T(*)[kWgK][kWgPitch]>(wg_lds);
  T(*Bs)[kWgK][kWgPitch] = As + 2;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 15, lg = lane >> 4;
  const int wi = wave >> 1, wj = wave & 1;
  const int tile = blockIdx.x;
  const int ti = tile / tj, tjx = tile % tj;
  const int ks = blockIdx.y;
  const long m0 = ks * rows_per;
  const long m1 = (m0 + rows_per < M) ? m0 + rows_per : M;
  const int i0 = ti * kWgTile, j0 = tjx * kWgTile;

  // copy slots: 16 rows x 128 columns per operand = 512 four-element units, two per thread
  int srow[2], scol[2];
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int u = tid + q * 256;
    srow[q] = u / 32;
    scol[q] = (u % 32) * 4;
  }
  v4 ra[2], rb[2];
  auto load_global = [&](long m) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const long row = m + srow[q];
      v4 za = {0, 0, 0, 0}, zb = {0, 0, 0, 0};
      if (row < m1) {
        if (i0 + scol[q] < ld_out) za = *reinterpret_cast<const v4 *>(Zb + row * ld_out + i0 + scol[q]);
        if (j0 + scol[q] < ld_in) zb = *reinterpret_cast<const v4 *>(H + row * ld_in + j0 + scol[q]);
      }
      ra[q] = za;
      rb[q] = zb;
    }
  };
  auto store_lds = [&](int st) {
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      *reinterpret_cast<v4 *>(&As[st][srow[q]][scol[q]]) = ra[q];
      *reinterpret_cast<v4 *>(&Bs[st][srow[q]][scol[q]]) = rb[q];
    }
  };

  vacc acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = vacc{0, 0, 0, 0};

  const long nst = (m1 - m0 + kWgK - 1) / kWgK;
  load_global(m0);
  store_lds(0);
  __syncthreads();
  for (long st = 0; st < nst; ++st) {
    const int cur = (int)(st & 1);
    if (st + 1 < nst) load_global(m0 + (st + 1) * kWgK);
#pragma unroll
    for (int kk = 0; kk < kWgK / 4; ++kk) {
      T af[4], bf[4];
#pragma unroll
      for (int a = 0; a < 4; ++a) af[a] = As[cur][kk * 4 + lg][wi * 64 + a * 16 + lr];
#pragma unroll
      for (int b = 0; b < 4; ++b) bf[b] = Bs[cur][kk * 4 + lg][wj * 64 + b * 16 + lr];
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = V::mfma(af[a], bf[b], acc[a][b]);
    }
    if (st + 1 < nst) store_lds(cur ^ 1);
    __syncthreads();
  }

  // partial tile -> partials[ks][i][j] (padded to whole tiles)
  const long pi = (long)gridDim.x / tj * kWgTile;  // padded rows
  const long pj = (long)tj * kWgTile;
  T *P = partials + (long)ks * pi * pj;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const long i = i0 + wi * 64 + a * 16 + V::out_row(lg, v);
        const long j = j0 + wj * 64 + b * 16 + lr;
        P[i * pj + j] = acc[a][b][v];
      }
}

// fp32 version with LDS-direct loads (global_load_lds_dwordx4, as in the stacked-GEMM kernel): a stage is [16 k][128
// features] per operand, unpadded (a wave instruction brings 1 KiB = two rows), two buffers.  Within a wave's 64 x 64
// block the MFMA row / column index l of block a stands for feature 4 l + a, so the four values a lane needs of one k row
// are 16 contiguous bytes: one ds_read_b128 per operand and k group (the 16 lanes of a quarter-wave read 256 contiguous
// bytes, conflict-free without any swizzle).  All addresses are a scalar base advanced by scalar adds plus constant
// per-lane offsets: the k loop holds LDS reads, MFMAs, the loads and one barrier per stage and no vector-ALU instruction
// (the guards and 64-bit address arithmetic of the generic kernel above cost its MFMA stream a fifth of its issue
// cycles).  Columns past the operand's width re-read column 0 of the tile: they only reach output entries the reduction
// never reads.  A ragged last stage (fewer than 16 rows) goes through registers with zero fill.
// TI = 128: a 128 x 128 output tile, waves 2 x 2.  TI = 256: 256 x 64, waves 4 x 1 (narrow inputs).
template <int TI>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 4)))
void wgrad_kernel_f32(const float *Zb, int ld_out, const float *H, int ld_in, long M, long rows_per, int tj, float *partials) {
  extern __shared__ __align__(16) unsigned char wg_lds[];
  constexpr int TJ = 128 * 128 / TI;                                // 128 or 64
  constexpr unsigned kRowA = TI * sizeof(float), kRowB = TJ * sizeof(float);   // LDS row pitches: 512 / 1024 and 512 / 256 B
  constexpr unsigned kOperandA = kWgK * kRowA, kOperandB = kWgK * kRowB;
  constexpr unsigned kBuffer = kOperandA + kOperandB;               // 16 or 20 KiB
  constexpr int kChunksA = kOperandA / 1024, kChunksB = kOperandB / 1024;      // 8 + 8 or 16 + 4 chunks of 1 KiB
  constexpr int NW = (kChunksA + kChunksB) / 4;                     // chunks per wave and stage: 4 or 5
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const int lr = lane & 15, lg = lane >> 4;
  const int wi = TI == 128 ? wave >> 1 : wave, wj = TI == 128 ? wave & 1 : 0;
  const int tile = blockIdx.x;
  const int ti = tile / tj, tjx = tile % tj;
  const int ks = blockIdx.y;
  const long m0 = ks * rows_per;
  const long m1 = (m0 + rows_per < M) ? m0 + rows_per : M;
  const int i0 = ti * TI, j0 = tjx * TJ;
  const int nfull = (int)((m1 - m0) / kWgK);    // rows_per is a multiple of 16 below 2^35
  const int tail = (int)((m1 - m0) - (long)nfull * kWgK);

  // ---- loads: a chunk is 1 KiB of a stage, i.e. 1024 / pitch whole rows; chunks 0 .. kChunksA-1 are Zbar, the others H;
  // wave w takes chunks w, w+4, ... (kChunksA is a multiple of 4, so position i of every wave is the same operand)
  unsigned c_voff[NW];
  unsigned c_lds[NW];
#pragma unroll
  for (int i = 0; i < NW; ++i) {
    const int c = wave_u + 4 * i;
    const bool isA = 4 * i < kChunksA;
    const int upr = (isA ? kRowA : kRowB) / 16;        // 16-byte units per row
    const int cidx = isA ? c : c - kChunksA;
    const int row = cidx * (64 / upr) + lane / upr;
    const int u = lane % upr;
    const int ld = isA ? ld_out : ld_in;
    const int c0 = isA ? i0 : j0;
    const int col = (c0 + u * 4 < ld) ? c0 + u * 4 : c0;
    c_voff[i] = (unsigned)(((long)row * ld + col) * sizeof(float));
    c_lds[i] = (isA ? 0u : kOperandA) + (unsigned)(cidx * 1024);
  }
  const unsigned lds_base = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char *)wg_lds;
  auto issue = [&](int buf, const float *ga, const float *gb) {   // ga, gb: first row of the stage in either operand (uniform)
#pragma unroll
    for (int i = 0; i < NW; ++i) {
      const unsigned off = lds_base + buf * kBuffer + c_lds[i];
      const float *g = 4 * i < kChunksA ? ga : gb;
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %2" : : "v"(c_voff[i]), "s"(off), "s"(g) : "memory");
    }
  };

  // ---- fragments: lane (lr, lg) reads features 4 lr .. 4 lr + 3 of k row 4 kk + lg of its wave's 64-feature strip
  const wf32x4 *Af = reinterpret_cast<const wf32x4 *>(wg_lds + lg * kRowA + wi * 256 + lr * 16);
  const wf32x4 *Bf = reinterpret_cast<const wf32x4 *>(wg_lds + kOperandA + lg * kRowB + wj * 256 + lr * 16);

  wf32x4 acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = wf32x4{0, 0, 0, 0};

  auto stage_mfmas = [&](int buf) {
#pragma unroll
    for (int kk = 0; kk < kWgK / 4; ++kk) {
      const wf32x4 af = Af[(buf * kBuffer + kk * 4 * kRowA) / 16], bf = Bf[(buf * kBuffer + kk * 4 * kRowB) / 16];
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[a], bf[b], acc[a][b], 0, 0, 0);
    }
  };

  if (nfull > 0) {
    const float *ga = Zb + m0 * ld_out, *gb = H + m0 * ld_in;
    const long sa = (long)kWgK * ld_out, sb = (long)kWgK * ld_in;
    issue(0, ga, gb);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    for (int st = 0; st < nfull; st += 2) {
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        if (half == 1 && st + 1 >= nfull) break;   // uniform
        // the other buffer was read during the previous stage, which ended with a barrier; the last stage re-fetches itself
        if (st + half + 1 < nfull) {
          ga += sa;
          gb += sb;
        }
        issue(half ^ 1, ga, gb);
        stage_mfmas(half);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's share of the next stage has landed
        __syncthreads();
      }
    }
  }
  if (tail > 0) {
    // fewer than 16 rows left: through registers, rows past the end are zeros.  Every wave passed the barrier that ends
    // the last full stage (and its surplus loads have landed), so buffer 0 is free.
    const long mt = m0 + (long)nfull * kWgK;
    constexpr int kUprA = kRowA / 16, kUprB = kRowB / 16;   // 16-byte units per row
#pragma unroll
    for (int q = 0; q < kWgK * kUprA / 256; ++q) {
      const int u4 = tid + q * 256;
      const int row = u4 / kUprA, u = u4 % kUprA;
      wf32x4 za = {0, 0, 0, 0};
      if (row < tail && i0 + u * 4 < ld_out) za = *reinterpret_cast<const wf32x4 *>(Zb + (mt + row) * ld_out + i0 + u * 4);
      *reinterpret_cast<wf32x4 *>(wg_lds + row * kRowA + u * 16) = za;
    }
#pragma unroll
    for (int q = 0; q < kWgK * kUprB / 256; ++q) {
      const int u4 = tid + q * 256;
      const int row = u4 / kUprB, u = u4 % kUprB;
      wf32x4 zb = {0, 0, 0, 0};
      if (row < tail && j0 + u * 4 < ld_in) zb = *reinterpret_cast<const wf32x4 *>(H + (mt + row) * ld_in + j0 + u * 4);
      *reinterpret_cast<wf32x4 *>(wg_lds + kOperandA + row * kRowB + u * 16) = zb;
    }
    __syncthreads();
    stage_mfmas(0);
  }

  // partial tile -> partials[ks][i][j] (padded to whole tiles)
  const long pi = (long)gridDim.x / tj * TI;  // padded rows
  const long pj = (long)tj * TJ;
  float *P = partials + (long)ks * pi * pj;
  // block (a, b), accumulator element v of lane (lr, lg) is output row 4 (4 lg + v) + a, column 4 lr + b of the wave's
  // 64 x 64 block: the four b of a lane are 16 contiguous bytes
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const long i = i0 + wi * 64 + (lg * 4 + v) * 4 + a;
      const long j = j0 + wj * 64 + lr * 4;
      *reinterpret_cast<wf32x4 *>(P + i * pj + j) = wf32x4{acc[a][0][v], acc[a][1][v], acc[a][2][v], acc[a][3][v]};
    }
}

// gW[i][j] = sum_k partials[k][i][j] in a fixed order: a block takes 64 outputs, its four wavefronts a quarter of
// the k range each (four running sums per thread keep several loads in flight), then the quarters are added.
template <typename T>
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const T *partials, int ksplit, long pi, long pj, int d_out, int d_in,
                                                           T *gW, int accumulate) {
  __shared__ T red[4][64];
  const int o = threadIdx.x & 63, g = threadIdx.x >> 6;
  const long total = (long)d_out * d_in;
  const long idx = blockIdx.x * 64L + o;
  T acc = T(0);
  if (idx < total) {
    const long i = idx / d_in, j = idx % d_in;
    const int per = (ksplit + 3) / 4;
    const int k0 = g * per, k1 = (k0 + per < ksplit) ? k0 + per : ksplit;
    const long stride = pi * pj;
    const T *p = partials + i * pj + j;
    T a0 = T(0), a1 = T(0), a2 = T(0), a3 = T(0);
    int k = k0;
    for (; k + 3 < k1; k += 4) {
      a0 += p[(long)k * stride];
      a1 += p[(long)(k + 1) * stride];
      a2 += p[(long)(k + 2) * stride];
      a3 += p[(long)(k + 3) * stride];
    }
    for (; k < k1; ++k) a0 += p[(long)k * stride];
    acc = (a0 + a1) + (a2 + a3);
  }
  red[g][o] = acc;
  __syncthreads();
  if (g == 0 && idx < total) {
    const T sum = (red[0][o] + red[1][o]) + (red[2][o] + red[3][o]);
    gW[idx] = accumulate ? gW[idx] + sum : sum;
  }
}

template <typename T>
hipError_t launch_wgrad(const T *Zbar, int ld_out, const T *H, int ld_in, long M, int d_out, int d_in, T *gW, T *partials,
                        hipStream_t s, int accumulate) {
  const WgradPlan p = wgrad_plan(M, d_out, d_in, wgrad_narrow(d_in, std::is_same<T, float>::value));
  if (p.ti * p.tj <= 0 || p.ksplit <= 0 || p.ksplit > 65535) return hipErrorInvalidValue;
  if constexpr (std::is_same<T, float>::value) {
    // 16-byte loads and stores: the operands and the partial sums must be 16-byte aligned (row pitches are multiples of 32 elements)
    if ((reinterpret_cast<size_t>(Zbar) | reinterpret_cast<size_t>(H) | reinterpret_cast<size_t>(partials)) & 15) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(p.ti * p.tj), (unsigned)p.ksplit);
    const size_t lds = 2 * (size_t)kWgK * (p.tile_i + p.tile_j) * sizeof(float);
    if (p.tile_i == kWgTile) {
      hipLaunchKernelGGL(wgrad_kernel_f32<128>, grid, dim3(256), lds, s, Zbar, ld_out, H, ld_in, M, p.rows_per, p.tj, partials);
    } else {
      hipLaunchKernelGGL(wgrad_kernel_f32<256>, grid, dim3(256), lds, s, Zbar, ld_out, H, ld_in, M, p.rows_per, p.tj, partials);
    }
  } else {
    constexpr size_t lds = 4 * (size_t)kWgK * kWgPitch * sizeof(T);
    static LdsLimitOnce lds_limit;
    hipError_t ea = lds_limit.ensure(reinterpret_cast<const void *>(&wgrad_kernel<T>), lds);
    if (ea != hipSuccess) return ea;
    hipLaunchKernelGGL(wgrad_kernel<T>, dim3((unsigned)(p.ti * p.tj), (unsigned)p.ksplit), dim3(256), lds, s, Zbar, ld_out, H, ld_in, M,
                       p.rows_per, p.tj, partials);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const long blocks = ((long)d_out * d_in + 63) / 64;
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(wgrad_reduce_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, s, partials, p.ksplit, (long)p.ti * p.tile_i,
                     (long)p.tj * p.tile_j, d_out, d_in, gW, accumulate);
  return hipGetLastError();
}
template hipError_t launch_wgrad<float>(const float *, int, const float *, int, long, int, int, float *, float *, hipStream_t, int);
template hipError_t launch_wgrad<double>(const double *, int, const double *, int, long, int, int, double *, double *, hipStream_t, int);

}  // namespace ctm
