// One-launch path for calls so small that launch latency is all there is to them: the whole propagation
// (Sec. 3.1, Eq. 6: seeds, every linear layer, the collapsed rule after each hidden layer, the last layer) runs in
// ONE workgroup, with the coefficient block of all points resident in LDS from the seeds to the outputs.
//
// Used when all N * rho coefficient rows fit 256 rows, the network is narrow and shallow enough for two coefficient
// blocks and all its weights to fit 64 KiB of LDS, and the handle computes in its storage type (fp64 / fp32).  The linear
// layers are plain dot products (k in ascending order, one fused multiply-add per term): with a few thousand
// multiply-adds per thread there is nothing for the matrix cores to win, and a launch costs more than the arithmetic.
// The rule is the same code as the stacked-GEMM epilogue (ctm_rule.h), applied in place to the pre-activations in LDS.
// Results therefore agree with the tiled path to rounding (different summation order in the dot products), and they
// do not depend on the rest of the batch: rows of different points never mix.
#include "ctm_internal.h"
#include "ctm_rule.h"

namespace ctm {

template <typename T> __global__ __launch_bounds__(256) void small_call_kernel(const SmallArgs<T> a) {
  // LDS: two coefficient blocks [rows][pitch], then every layer's weights (hidden layers transposed, [d_in][d_out], so that
  // the threads of a row read consecutive words) and biases -- all staged once at the start, so the call waits for global memory once
  extern __shared__ __align__(16) unsigned char small_lds[];
  T *lds = reinterpret_cast<T *>(small_lds);
  const int rows = a.N * a.rho;
  const int pitch = a.pitch;
  const int blk = rows * pitch;          // elements per coefficient block
  const int tid = threadIdx.x;
  const int L = a.L;

  int woff[kSmallMaxLayers], boff[kSmallMaxLayers];
  {
    int off = 2 * blk;
    for (int l = 0; l < L; ++l) {
      woff[l] = off;
      off += a.dims[l] * a.dims[l + 1];
      boff[l] = off;
      off += a.dims[l + 1];
    }
  }
  for (int l = 0; l < L; ++l) {
    const int din = a.dims[l], dout = a.dims[l + 1], ldw = a.ld[l];
    const T *W = a.W[l];                 // packed [>= dout][ldw]
    T *Ws = lds + woff[l];
    for (int j = tid; j < dout; j += 256) lds[boff[l] + j] = a.b[l][j];
    if (l + 1 < L) {
      for (int i = tid; i < din * dout; i += 256) {
        const int k = i % din, j = i / din;
        Ws[k * dout + j] = W[(long)j * ldw + k];
      }
    } else {
      for (int i = tid; i < din * dout; i += 256) Ws[i] = W[(long)(i / din) * ldw + i % din];   // [C][d_{L-1}]
    }
  }
  // seeds (Sec. 3.1): row 0 of a point is x_n, its first-order rows are the directions, every other row is zero
  {
    const int D = a.dims[0];
    for (int i = tid; i < rows * D; i += 256) {
      const int k = i % D, row = i / D;
      const int c = row % a.rho, n = row / a.rho;
      T v = T(0);
      if (c == 0) {
        v = a.x[(long)n * D + k];
      } else if (c < a.rho - 1) {
        int r = -1;
        if (a.order == 2) r = c - 1;
        else if ((c - 1) % 3 == 0) r = (c - 1) / 3;
        if (r >= 0) v = a.V ? a.V[n * a.v_sn + r * a.v_sr + k * a.v_sd] : (k == r ? T(1) : T(0));
      }
      lds[row * pitch + k] = v;
    }
  }
  __syncthreads();

  LayerArgs<T> la = {};
  la.R = a.R; la.act = a.act; la.order = a.order; la.standard = 0; la.rho = a.rho;
  int in_off = 0, out_off = blk;
  for (int l = 0; l + 1 < L; ++l) {
    const int din = a.dims[l], dout = a.dims[l + 1];
    const T *Ws = lds + woff[l];
    for (int i = tid; i < rows * dout; i += 256) {
      const int j = i % dout, row = i / dout;
      const T *h = lds + in_off + row * pitch;
      T z = T(0);
      int k = 0;
      for (; k + 3 < din; k += 4) {   // four terms' operands fetched together, added in ascending k
        const T h0 = h[k], h1 = h[k + 1], h2 = h[k + 2], h3 = h[k + 3];
        const T w0 = Ws[k * dout + j], w1 = Ws[(k + 1) * dout + j], w2 = Ws[(k + 2) * dout + j], w3 = Ws[(k + 3) * dout + j];
        z += h0 * w0; z += h1 * w1; z += h2 * w2; z += h3 * w3;
      }
      for (; k < din; ++k) z += h[k] * Ws[k * dout + j];
      lds[out_off + row * pitch + j] = z;
    }
    __syncthreads();
    // the rule, in place: one thread per (point, feature) walks the point's rows; a row is read before it is overwritten
    la.last = (l == L - 2) ? 1 : 0;
    const T *bias = lds + boff[l];
    for (int i = tid; i < a.N * dout; i += 256) {
      const int j = i % dout, p = i / dout;
      T *col = lds + out_off + p * a.rho * pitch;
      jet_rule<T, PlainRows<T>, 1, false>(col + j, pitch, bias[j], PlainRows<T>{col, pitch, (unsigned)(j * sizeof(T))}, la);
    }
    __syncthreads();
    const int t = in_off; in_off = out_off; out_off = t;
  }

  // last layer (App. H: linear, bias on the order-0 coefficient only): rows 0 and 1 of a point hold h_0 and h_K
  const int dl = a.dims[L - 1];
  const T *w = lds + woff[L - 1];
  for (int i = tid; i < a.N * a.C; i += 256) {
    const int c = i % a.C, n = i / a.C;
    const T *h0 = lds + in_off + n * a.rho * pitch;
    T s0 = T(0), sk = T(0);
    for (int k = 0; k < dl; ++k) {
      const T wk = w[c * dl + k];
      s0 += wk * h0[k];
      sk += wk * h0[pitch + k];
    }
    const T opv = (T)(a.scale * (double)sk);
    if (a.accumulate) {
      if (a.op) a.op[i] += opv;
    } else {
      if (a.u) a.u[i] = s0 + lds[boff[L - 1] + c];
      if (a.op) a.op[i] = opv;
    }
  }
}

// widest layer + 1: a row pitch that is not a multiple of the bank count keeps the rows of a column in different LDS banks
int small_call_pitch(const int *dims, int L) {
  int dmax = 0;
  for (int l = 0; l < L; ++l) dmax = dims[l] > dmax ? dims[l] : dmax;
  return dmax + 1;
}

size_t small_call_lds_bytes(const int *dims, int L, long rows, size_t elem_size) {
  size_t w = 0;
  for (int l = 0; l < L; ++l) w += (size_t)(dims[l] + 1) * dims[l + 1];   // weights and biases
  return (2 * (size_t)rows * small_call_pitch(dims, L) + w) * elem_size;
}

template <typename T> hipError_t launch_small_call(const SmallArgs<T> &a, size_t lds_bytes, hipStream_t s) {
  if (lds_bytes > kSmallMaxLds || (long)a.N * a.rho > kSmallMaxRows || a.L > kSmallMaxLayers) return hipErrorInvalidValue;
  hipLaunchKernelGGL(small_call_kernel<T>, dim3(1), dim3(256), lds_bytes, s, a);
  return hipGetLastError();
}
template hipError_t launch_small_call<float>(const SmallArgs<float> &, size_t, hipStream_t);
template hipError_t launch_small_call<double>(const SmallArgs<double> &, size_t, hipStream_t);

}  // namespace ctm
