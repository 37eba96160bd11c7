// First layer for direction sets shared by all points (standard basis, shared V, sigma).
//
// With seeds x_{0} = x_n, x_{1,r} = v_r, x_{k>=2} = 0 (Sec. 3.1) the first linear layer gives
//   z_0(n) = W_1 x_n + b_1          -- one small dot product per (point, feature)
//   z_{1,r} = W_1 v_r               -- the same for every point, so it is computed once
//   z_{k>=2} = 0
// and the activation rule (same formulas as in the stacked-GEMM epilogue) reduces to products
// of per-(point, feature) factors with per-(direction, feature) constants:
//   order 2:  h_0 = t, h_{1,r} = d1 * z1_r, h_2 = d2 * sum_r z1_r^2
//   order 4:  h_{1,r} = d1 z1_r, h_{2,r} = d2 z1_r^2, h_{3,r} = d3 z1_r^3, h_4 = d4 * sum_r z1_r^4
// so the whole layer is bound by writing the [N * rho, d_1] block to HBM; no GEMM over the
// rho rows of every point is needed.
#include "ctm_internal.h"
#include "ctm_rule.h"

#include <type_traits>

namespace ctm {

// z1[r][j] = sum_k W[j][k] v_r[k] for an explicit direction set V.  One thread per (direction, feature).
// (For the standard basis z1[r] is row r of the transposed weights and the first-layer kernel reads it there.)
template <typename T> __global__ void first_dirs_kernel(const FirstArgs<T> a) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  const int r = blockIdx.y;
  if (j >= a.ld1) return;
  const T *w = a.WT + j;   // W_1 transposed: consecutive threads read consecutive words
  const long ws = a.ld1;
  const T *v = a.V + (long)(a.r0 + r) * a.v_sr;
  T z = T(0);
  int k = 0;
  for (; k + 7 < a.D; k += 8) {   // eight terms' operands in flight at once; k ascending
    T wv[8], vv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) { wv[i] = w[(k + i) * ws]; vv[i] = v[(long)(k + i) * a.v_sd]; }
#pragma unroll
    for (int i = 0; i < 8; ++i) z += wv[i] * vv[i];
  }
  for (; k < a.D; ++k) z += w[k * ws] * v[(long)k * a.v_sd];
  a.Z1[(long)r * a.ld1 + j] = z;
}

constexpr int kFirstPoints = 16;      // points per workgroup ...
constexpr int kFirstPointsSmall = 4;  // ... and in batches too small to give every compute unit two such workgroups
constexpr int kFirstDmax = 64;        // input widths up to this are held in registers

// BF = 0: out holds rows of T; BF = 1: out is written as bf16 (input of the plain-bf16 GEMM kernel).
// DM: the input width rounded up to 8, 16, 32 or 64 -- the length of the register-resident weight row and of the dot
// products (a 5-dimensional problem should not pay for 64 inputs).  NP: points per workgroup.
// A thread's weight row comes from the transposed copy of W_1, so that the threads of a wavefront read consecutive
// words (from the row-major copy every lane would open a cache line of its own for each of its D words).
template <typename T, int BF, int DM, int NP> __global__ __launch_bounds__(256) void first_layer_kernel(const FirstArgs<T> a) {
  __shared__ T xs[NP][DM];
  const int tid = threadIdx.x;
  const int j = blockIdx.x * 256 + tid;
  const long n0 = (long)blockIdx.y * NP;
  const int np = (int)((a.N - n0) < NP ? (a.N - n0) : NP);
  for (int i = tid; i < NP * DM; i += 256) {  // unused entries must be zero, not stale
    const int p = i / DM, k = i % DM;
    xs[p][k] = (p < np && k < a.D) ? a.x[(n0 + p) * a.D + k] : T(0);
  }
  __syncthreads();
  if (j >= a.ld1) return;

  T w[DM];
#pragma unroll
  for (int k = 0; k < DM; ++k) w[k] = k < a.D ? a.WT[(long)k * a.ld1 + j] : T(0);
  const T bias = a.bias[j];

  T t[NP], d1[NP];
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    t[p] = d1[p] = T(0);
    if (p < np) {   // uniform: a short last chunk (or a tiny batch) skips the activations of absent points
      T z0 = bias;
#pragma unroll
      for (int k = 0; k < DM; ++k) z0 += w[k] * xs[p][k];   // k >= D: both factors are zero
      act_eval<T>(a.act, z0, t[p], d1[p]);
    }
  }

  const long ld = a.ld1;
  const int rho = a.rho;
  const long obase = ((a.out_point0 + n0) * a.out_rows) * ld + j;
  const long pstep = (long)a.out_rows * ld;
  auto put = [&](long off, T v) {  // off: element offset from this thread's first output element
    if constexpr (BF == 0) {
      a.out[obase + off] = v;
    } else {
      reinterpret_cast<__bf16 *>(a.out)[obase + off] = (__bf16)(float)v;
    }
  };
#pragma unroll
  for (int p = 0; p < NP; ++p)
    if (p < np) put(p * pstep, t[p]);
  T mom = T(0);  // sum_r z1_r^order, the only term of the collapsed row at the first layer
  for (int r = 0; r < a.R; ++r) {
    const T z1 = a.Z1[(long)r * ld + j];
    const T z1s = z1 * z1;
    mom += (a.order == 2) ? z1s : z1s * z1s;
    if (a.standard) {
      // un-collapsed layout: every direction has its own highest-order row, d_K * z1^K at this layer
      const T zK = (a.order == 2) ? z1s : z1s * z1s;
      const int K = a.order;
      const long row1 = (K == 2) ? 1 + r : 1 + 4 * r;            // first-order row of direction r
      const long rowK = a.last ? 1 + r : ((K == 2) ? 1 + a.R + r : 4 + 4 * r);
#pragma unroll
      for (int p = 0; p < NP; ++p)
        if (p < np) {
          const T d2 = act_d2<T>(a.act, t[p], d1[p]);
          const T dK = (K == 2) ? d2 : act_d4<T>(a.act, t[p], d1[p]);
          put(p * pstep + rowK * ld, dK * zK);
          if (!a.last) {
            put(p * pstep + row1 * ld, d1[p] * z1);
            if (K == 4) {
              const T d3 = act_d3<T>(a.act, t[p], d1[p]);
              put(p * pstep + (row1 + 1) * ld, d2 * z1s);
              put(p * pstep + (row1 + 2) * ld, d3 * z1s * z1);
            }
          }
        }
      continue;
    }
    if (a.last) continue;
    if (a.order == 2) {
      const long orow = (long)(1 + r) * ld;
#pragma unroll
      for (int p = 0; p < NP; ++p)
        if (p < np) put(orow + p * pstep, d1[p] * z1);
    } else {
      const long orow = (long)(1 + 3 * r) * ld;
      const T z1c = z1s * z1;
#pragma unroll
      for (int p = 0; p < NP; ++p)
        if (p < np) {
          const T d2 = act_d2<T>(a.act, t[p], d1[p]), d3 = act_d3<T>(a.act, t[p], d1[p]);
          put(orow + p * pstep, d1[p] * z1);
          put(orow + p * pstep + ld, d2 * z1s);
          put(orow + p * pstep + 2 * ld, d3 * z1c);
        }
    }
  }
  if (a.standard) return;  // no collapsed row
  const long olast = (long)(a.last ? 1 : rho - 1) * ld;
#pragma unroll
  for (int p = 0; p < NP; ++p)
    if (p < np) {
      const T dk = (a.order == 2) ? act_d2<T>(a.act, t[p], d1[p]) : act_d4<T>(a.act, t[p], d1[p]);
      put(olast + p * pstep, dk * mom);
    }
}

// ---- per-point directions in a low-dimensional input space (D <= 16) ------------------------------------------
// z_{1,r}(n) = W_1 v_{n,r} differs from point to point, but with so few inputs it is cheaper as D multiply-adds per
// (row, feature) than as a stacked GEMM over a seeded block whose higher-order rows are all zero: the layer is then
// bound by writing its output block, like the shared-direction kernel above.  A workgroup takes kPPPoints points;
// their x and directions are staged in LDS (zero-padded to 16 inputs) and read back 4 inputs at a time.
constexpr int kPPPoints = 2;  // measured on the order-4 benchmark workload: 1 -> 26 us, 2 -> 28 us, 4 -> 44 us (too few workgroups);
                              // sharing a point's directions out over four workgroups (each recomputing the moment): 42 us
constexpr int kPPDmax = 16;

template <typename T, int BF> __global__ __launch_bounds__(256) void first_layer_pp_kernel(const FirstArgs<T> a) {
  extern __shared__ __align__(16) unsigned char pp_lds[];
  T *xs = reinterpret_cast<T *>(pp_lds);                 // [kPPPoints][16]
  T *vs = xs + kPPPoints * kPPDmax;                      // [kPPPoints][R][16]
  const int tid = threadIdx.x;
  const int j = blockIdx.y * 256 + tid;                  // blockIdx.x runs over the points (it has the larger range)
  const long n0 = (long)blockIdx.x * kPPPoints;
  const int np = (int)((a.N - n0) < kPPPoints ? (a.N - n0) : kPPPoints);
  const int R = a.R;
  for (int i = tid; i < kPPPoints * kPPDmax; i += 256) {
    const int p = i / kPPDmax, k = i % kPPDmax;
    xs[i] = (p < np && k < a.D) ? a.x[(n0 + p) * a.D + k] : T(0);
  }
  for (int i = tid; i < kPPPoints * R * kPPDmax; i += 256) {
    const int k = i % kPPDmax;
    const int r = (i / kPPDmax) % R;
    const int p = i / (kPPDmax * R);
    vs[i] = (p < np && k < a.D) ? a.V[(n0 + p) * a.v_sn + (long)(a.r0 + r) * a.v_sr + (long)k * a.v_sd] : T(0);
  }
  __syncthreads();
  if (j >= a.ld1) return;

  T w[kPPDmax];
#pragma unroll
  for (int k = 0; k < kPPDmax; ++k) w[k] = k < a.D ? a.W[(long)j * a.ld0 + k] : T(0);
  const T bias = a.bias[j];
  const long ld = a.ld1;
  const int rho = a.rho, K = a.order;
  auto dot16 = [&](const T *v) {   // v: 16 staged inputs, the same address for every lane (LDS broadcast reads)
    T acc = T(0);
#pragma unroll
    for (int k = 0; k < kPPDmax; ++k) acc += w[k] * v[k];
    return acc;
  };
  for (int p = 0; p < np; ++p) {
    const long obase = ((a.out_point0 + n0 + p) * a.out_rows) * ld + j;
    auto put = [&](long row, T v) {
      if constexpr (BF == 0) a.out[obase + row * ld] = v;
      else reinterpret_cast<__bf16 *>(a.out)[obase + row * ld] = (__bf16)(float)v;
    };
    T t, d1;
    act_eval<T>(a.act, bias + dot16(xs + p * kPPDmax), t, d1);
    const T d2 = act_d2<T>(a.act, t, d1);
    const T d3 = K == 4 ? act_d3<T>(a.act, t, d1) : T(0);
    const T dK = K == 2 ? d2 : act_d4<T>(a.act, t, d1);
    put(0, t);
    T mom = T(0);  // sum_r z1_r^K, the only term of the collapsed row at the first layer
    int r = 0;
    if (!a.standard && !a.last) {
      // four directions per trip: their dot products are independent chains of multiply-adds, and their stores go out
      // together; the moment still adds the directions in ascending order
      for (; r + 3 < R; r += 4) {
        T z[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) z[i] = dot16(vs + ((long)p * R + r + i) * kPPDmax);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const T z1 = z[i], z1s = z1 * z1;
          mom += K == 2 ? z1s : z1s * z1s;
          if (K == 2) {
            put(1 + r + i, d1 * z1);
          } else {
            put(1 + 3 * (r + i), d1 * z1);
            put(2 + 3 * (r + i), d2 * z1s);
            put(3 + 3 * (r + i), d3 * z1s * z1);
          }
        }
      }
    }
    for (; r < R; ++r) {
      const T z1 = dot16(vs + ((long)p * R + r) * kPPDmax);
      const T z1s = z1 * z1;
      const T zK = K == 2 ? z1s : z1s * z1s;
      mom += zK;
      if (a.standard) {  // un-collapsed layout: direction r keeps its own highest-order row, d_K z1^K at this layer
        const long row1 = K == 2 ? 1 + r : 1 + 4 * r;
        const long rowK = a.last ? 1 + r : (K == 2 ? 1 + R + r : 4 + 4 * r);
        put(rowK, dK * zK);
        if (!a.last) {
          put(row1, d1 * z1);
          if (K == 4) {
            put(row1 + 1, d2 * z1s);
            put(row1 + 2, d3 * z1s * z1);
          }
        }
      } else if (!a.last) {
        if (K == 2) {
          put(1 + r, d1 * z1);
        } else {
          put(1 + 3 * r, d1 * z1);
          put(2 + 3 * r, d2 * z1s);
          put(3 + 3 * r, d3 * z1s * z1);
        }
      }
    }
    if (!a.standard) put(a.last ? 1 : rho - 1, dK * mom);
  }
}

// 0: no fast path (seed block + stacked GEMM); 1: shared directions; 2: per-point directions, D <= 16
int first_layer_fast_path(int D, long v_point_stride, int R) {
  if (v_point_stride == 0) return D <= kFirstDmax ? 1 : 0;
  const size_t lds = (size_t)kPPPoints * (1 + (size_t)R) * kPPDmax * sizeof(double);
  return (D <= kPPDmax && lds <= 96 * 1024) ? 2 : 0;
}

template <typename T> static hipError_t launch_first_pp(const FirstArgs<T> &a, hipStream_t s) {
  const size_t lds = (size_t)kPPPoints * (1 + (size_t)a.R) * kPPDmax * sizeof(T);
  const long chunks = (a.N + kPPPoints - 1) / kPPPoints;
  if (chunks > 0x7fffffffL || (a.ld1 + 255) / 256 > 65535) return hipErrorInvalidValue;
  static LdsLimitOnce lim0, lim1;
  hipError_t e = lim0.ensure(reinterpret_cast<const void *>(&first_layer_pp_kernel<T, 0>), 96 * 1024);
  if (e != hipSuccess) return e;
  if constexpr (std::is_same<T, float>::value) {
    e = lim1.ensure(reinterpret_cast<const void *>(&first_layer_pp_kernel<T, 1>), 96 * 1024);
    if (e != hipSuccess) return e;
  }
  const dim3 grid((unsigned)chunks, (a.ld1 + 255) / 256);
  bool launched = false;
  if constexpr (std::is_same<T, float>::value) {
    if (a.out_bf16) { hipLaunchKernelGGL((first_layer_pp_kernel<T, 1>), grid, dim3(256), lds, s, a); launched = true; }
  }
  if (!launched) {
    if (a.out_bf16) return hipErrorInvalidValue;
    hipLaunchKernelGGL((first_layer_pp_kernel<T, 0>), grid, dim3(256), lds, s, a);
  }
  return hipGetLastError();
}

template <typename T, int DM, int NP> static hipError_t launch_first_dm(const FirstArgs<T> &b, dim3 grid, hipStream_t s) {
  if constexpr (std::is_same<T, float>::value) {
    if (b.out_bf16) {
      hipLaunchKernelGGL((first_layer_kernel<T, 1, DM, NP>), grid, dim3(256), 0, s, b);
      return hipGetLastError();
    }
  }
  if (b.out_bf16) return hipErrorInvalidValue;
  hipLaunchKernelGGL((first_layer_kernel<T, 0, DM, NP>), grid, dim3(256), 0, s, b);
  return hipGetLastError();
}
template <typename T, int NP> static hipError_t launch_first_width(const FirstArgs<T> &b, dim3 grid, hipStream_t s) {
  if (b.D > kFirstDmax) return hipErrorInvalidValue;
  if (b.D <= 8) return launch_first_dm<T, 8, NP>(b, grid, s);
  if (b.D <= 16) return launch_first_dm<T, 16, NP>(b, grid, s);
  if (b.D <= 32) return launch_first_dm<T, 32, NP>(b, grid, s);
  return launch_first_dm<T, 64, NP>(b, grid, s);
}

template <typename T> hipError_t launch_first(const FirstArgs<T> &a, hipStream_t s) {
  if (a.v_sn != 0) return launch_first_pp<T>(a, s);
  hipError_t e = hipSuccess;
  FirstArgs<T> dirs = a;
  if (a.V == nullptr) {
    // standard basis: W_1 e_r is row r of the transposed weights, nothing to compute (the kernel only reads Z1)
    dirs.Z1 = const_cast<T *>(a.WT) + (long)a.r0 * a.ld1;
  } else {
    hipLaunchKernelGGL(first_dirs_kernel<T>, dim3((a.ld1 + 255) / 256, a.R), dim3(256), 0, s, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  // 16 points per workgroup amortise the weight row best; a batch that gives fewer than two such workgroups per compute
  // unit is latency-bound instead and takes 4 (sigma-weighted Laplacian, N = 2048: 41 -> 29 us with the transposed reads).
  // The arithmetic of a (point, feature) pair is the same either way.
  const long col_blocks = (a.ld1 + 255) / 256;
  const bool small = ((a.N + kFirstPoints - 1) / kFirstPoints) * col_blocks < 2L * a.cus;
  const int np = small ? kFirstPointsSmall : kFirstPoints;
  const long chunks = (a.N + np - 1) / np;
  if (chunks > 65535L * 65535L) return hipErrorInvalidValue;
  // grid.y is limited to 65535: fold larger batches into several launches
  for (long c0 = 0; c0 < chunks; c0 += 65535) {
    const long nc = (chunks - c0) < 65535 ? (chunks - c0) : 65535;
    FirstArgs<T> b = dirs;
    b.x = a.x + c0 * np * a.D;
    b.out_point0 = c0 * np;
    b.N = a.N - c0 * np;
    if (b.N > nc * np) b.N = nc * np;
    const dim3 grid((unsigned)col_blocks, (unsigned)nc);
    e = small ? launch_first_width<T, kFirstPointsSmall>(b, grid, s) : launch_first_width<T, kFirstPoints>(b, grid, s);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}
template hipError_t launch_first<float>(const FirstArgs<float> &, hipStream_t);
template hipError_t launch_first<double>(const FirstArgs<double> &, hipStream_t);

}  // namespace ctm
