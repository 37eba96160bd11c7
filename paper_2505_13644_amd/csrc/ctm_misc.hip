// Small bandwidth-bound kernels around the stacked GEMM: seeding the input coefficient
// block, re-packing weights at handle creation, and the last (width-1) linear layer.
#include "ctm_internal.h"

#include <type_traits>

namespace ctm {

// ---- input jets (Sec. 3.1: x_{0,r} = x_0, x_{1,r} = v_r, x_{k>=2,r} = 0) ---------------
// Row c of point n:  c = 0 -> x_n ; first-order rows -> v_r ; every other row -> 0.
// order 2: rows 1..R are first order.  order 4: rows 1+3r are first order, 2+3r and 3+3r are
// the (zero) second and third order coefficients of direction r.
template <typename T> __global__ void seed_kernel(const SeedArgs<T> a) {
  const long total = a.N * a.rho * a.ld;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const int k = (int)(i % a.ld);
    const long m = i / a.ld;
    const int c = (int)(m % a.rho);
    const long n = m / a.rho;
    T v = T(0);
    if (k < a.D) {
      if (c == 0) {
        v = a.x[n * a.D + k];
      } else if (a.standard || c < a.rho - 1) {
        int r = -1;
        if (a.standard) {  // order 2: rows 1..R; order 4: rows 1 + 4r
          if (a.order == 2) r = c <= a.R ? c - 1 : -1;
          else if ((c - 1) % 4 == 0) r = (c - 1) / 4;
        } else if (a.order == 2) r = c - 1;
        else if ((c - 1) % 3 == 0) r = (c - 1) / 3;
        if (r >= 0) {
          r += a.r0;
          v = a.V ? a.V[n * a.v_sn + r * a.v_sr + k * a.v_sd] : (k == r ? T(1) : T(0));
        }
      }
    }
    if constexpr (std::is_same<T, float>::value) {
      if (a.out_bf16) {
        reinterpret_cast<__bf16 *>(a.out)[i] = (__bf16)v;
        continue;
      }
    }
    a.out[i] = v;
  }
}

template <typename T> hipError_t launch_seed(const SeedArgs<T> &a, hipStream_t s) {
  const long total = a.N * a.rho * a.ld;
  long blocks = (total + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(seed_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}
template hipError_t launch_seed<float>(const SeedArgs<float> &, hipStream_t);
template hipError_t launch_seed<double>(const SeedArgs<double> &, hipStream_t);

// ---- weights: [d_out][d_in] -> zero-padded [rows_pad][ld]; bias -> [rows_pad] ---------------
template <typename T>
__global__ void pack_kernel(const T *W, const T *b, int d_out, int d_in, T *Wp, T *bp, int rows_pad, int ld, int transpose) {
  const long total = (long)rows_pad * ld;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const int k = (int)(i % ld);
    const int j = (int)(i / ld);
    T v = T(0);
    if (j < d_out && k < d_in) v = transpose ? W[(long)k * d_out + j] : W[(long)j * d_in + k];
    Wp[i] = v;
    if (k == 0 && bp != nullptr) bp[j] = (b != nullptr && j < d_out) ? b[j] : T(0);
  }
}

template <typename T>
hipError_t launch_pack(const T *W, const T *b, int d_out, int d_in, T *Wp, T *bp, int rows_pad, int ld, hipStream_t s,
                       int transpose) {
  const long total = (long)rows_pad * ld;
  long blocks = (total + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(pack_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, s, W, b, d_out, d_in, Wp, bp, rows_pad, ld, transpose);
  return hipGetLastError();
}
template hipError_t launch_pack<float>(const float *, const float *, int, int, float *, float *, int, int, hipStream_t, int);
template hipError_t launch_pack<double>(const double *, const double *, int, int, double *, double *, int, int, hipStream_t, int);

// ---- direction sets of the exact biharmonic (Sec. 3.3 / App. E.1: 4-jets along 4 e_d, 3 e_d1 + e_d2, 2 e_d1 + 2 e_d2)
template <typename T> __global__ void biharm_dirs_kernel(T *V, int D, int family, long rows) {
  const long total = rows * D;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const int k = (int)(i % D);
    const long r = i / D;
    T v = T(0);
    if (family == 0) {
      v = (k == r) ? T(4) : T(0);
    } else if (family == 1) {  // r enumerates (d1, d2) with d2 != d1: d2 skips d1
      const int d1 = (int)(r / (D - 1));
      int d2 = (int)(r % (D - 1));
      d2 += d2 >= d1 ? 1 : 0;
      v = (k == d1) ? T(3) : (k == d2 ? T(1) : T(0));
    } else {  // r enumerates pairs d1 < d2 in lexicographic order
      long rem = r;
      int d1 = 0;
      while (rem >= D - 1 - d1) { rem -= D - 1 - d1; ++d1; }
      const int d2 = d1 + 1 + (int)rem;
      v = (k == d1 || k == d2) ? T(2) : T(0);
    }
    V[i] = v;
  }
}

template <typename T> hipError_t launch_biharm_dirs(T *V, int D, int family, hipStream_t s) {
  const long rows = family == 0 ? D : (family == 1 ? (long)D * (D - 1) : (long)D * (D - 1) / 2);
  if (rows == 0) return hipSuccess;
  long blocks = (rows * D + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(biharm_dirs_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, s, V, D, family, rows);
  return hipGetLastError();
}
template hipError_t launch_biharm_dirs<float>(float *, int, int, hipStream_t);
template hipError_t launch_biharm_dirs<double>(double *, int, int, hipStream_t);

// ---- directions of the stochastic weighted Laplacian (Sec. 3.2, Eq. 8, stochastic case): sigma_n v_{n,s}
template <typename T>
__global__ void sigma_dirs_kernel(const T *sigma, long sig_stride, const T *V, long v_stride, T *out, long Nd, int S, int D, int K) {
  const long total = Nd * S * D;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const int d = (int)(i % D);
    const long ns = i / D;
    const int sidx = (int)(ns % S);
    const long n = ns / S;
    const T *sg = sigma + n * sig_stride + (long)d * K;
    const T *v = V + n * v_stride + (long)sidx * K;
    T acc = T(0);
    for (int k = 0; k < K; ++k) acc += sg[k] * v[k];
    out[i] = acc;
  }
}

template <typename T>
hipError_t launch_sigma_dirs(const T *sigma, long sig_stride, const T *V, long v_stride, T *out, long Nd, int S, int D, int K,
                             hipStream_t s) {
  long blocks = (Nd * S * D + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(sigma_dirs_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, s, sigma, sig_stride, V, v_stride, out, Nd, S, D, K);
  return hipGetLastError();
}
template hipError_t launch_sigma_dirs<float>(const float *, long, const float *, long, float *, long, int, int, int, hipStream_t);
template hipError_t launch_sigma_dirs<double>(const double *, long, const double *, long, double *, long, int, int, int, hipStream_t);

// ---- last layer (App. H: g is linear, bias on the 0-th coefficient only) ------------------
//   u_{n,c} = w_c . h_0(n) + b_c        op_{n,c} = scale * (w_c . h_K(n))       (Sec. 3.2: one operator value per output)
// One wavefront per point; lanes stride the features, outputs are taken four at a time, and the 64
// partial sums are folded with a fixed butterfly, so the result does not depend on scheduling.
template <typename T> __global__ __launch_bounds__(256) void final_kernel(const FinalArgs<T> a) {
  const int lane = threadIdx.x & 63;
  const long n = blockIdx.x * 4L + (threadIdx.x >> 6);
  if (n >= a.N) return;
  const T *h0 = a.pair + n * (1 + a.nk) * a.ld;
  for (int c0 = 0; c0 < a.C; c0 += 4) {
    T s0[4] = {T(0), T(0), T(0), T(0)}, sk[4] = {T(0), T(0), T(0), T(0)};
    const int nc = (a.C - c0) < 4 ? (a.C - c0) : 4;   // outputs of this group (uniform); unused slots stay zero
    // kU strides of the feature loop at a time: all their loads are issued before the first multiply-add, which are
    // then taken in ascending k as before (one stride at a time the loop paid a memory round trip per 64 features)
    constexpr int kU = 4;
    for (int kb = lane; kb < a.ld; kb += 64 * kU) {
      T v0[kU], hk[kU], wv[kU][4];
#pragma unroll
      for (int q = 0; q < kU; ++q) {
        const int k = kb + 64 * q;
        const bool in = k < a.ld;
        v0[q] = in ? h0[k] : T(0);
        hk[q] = T(0);
        if (in)
          for (int r = 1; r <= a.nk; ++r) hk[q] += h0[(long)r * a.ld + k];  // nk > 1: the sum un-collapsed mode defers to the end
#pragma unroll
        for (int i = 0; i < 4; ++i) wv[q][i] = (in && i < nc) ? a.w[(long)(c0 + i) * a.ld + k] : T(0);
      }
#pragma unroll
      for (int q = 0; q < kU; ++q) {
        if (kb + 64 * q < a.ld) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            if (i < nc) {
              s0[i] += wv[q][i] * v0[q];
              sk[i] += wv[q][i] * hk[q];
            }
          }
        }
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (i < nc) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
          s0[i] += __shfl_xor(s0[i], off, 64);
          sk[i] += __shfl_xor(sk[i], off, 64);
        }
      }
    }
    if (lane == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int c = c0 + i;
        if (c >= a.C) break;
        const T opv = (T)(a.scale * (double)sk[i]);
        const long o = n * a.C + c;
        if (a.accumulate) {
          if (a.op) a.op[o] += opv;
        } else {
          if (a.u) a.u[o] = s0[i] + a.b[c];
          if (a.op) a.op[o] = opv;
        }
      }
    }
  }
}

template <typename T> hipError_t launch_final(const FinalArgs<T> &a, hipStream_t s) {
  const long blocks = (a.N + 3) / 4;
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(final_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}
template hipError_t launch_final<float>(const FinalArgs<float> &, hipStream_t);
template hipError_t launch_final<double>(const FinalArgs<double> &, hipStream_t);

}  // namespace ctm
