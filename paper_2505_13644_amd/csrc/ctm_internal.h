// Internal declarations shared by the translation units of libctm.so.
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <cstddef>

namespace ctm {

// Raises a kernel's dynamic-LDS limit the first time it is launched on each device (the attribute belongs to
// the device's copy of the kernel); safe to call from several threads.
struct LdsLimitOnce {
  std::atomic<unsigned long long> done{0};
  hipError_t ensure(const void *kernel, size_t bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const bool tracked = dev >= 0 && dev < 64;
    if (tracked && ((done.load(std::memory_order_acquire) >> dev) & 1ull)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess && tracked) done.fetch_or(1ull << dev, std::memory_order_release);
    return e;
  }
};

// Shape constants of the stacked-GEMM kernel, per storage type.
//   KV  elements per 16-byte LDS/global vector
//   BK  K-extent of one LDS stage (4 * KV: each lane's 16-byte fragment feeds KV MFMAs)
//   NB  16-column MFMA blocks per wave; a workgroup has 4 waves side by side
template <typename T> struct Shape;
template <> struct Shape<float> {
  static constexpr int KV = 4, BK = 16, NB = 2;
};
template <> struct Shape<double> {
  static constexpr int KV = 2, BK = 8, NB = 1;
};
template <typename T> constexpr int tile_cols() { return 64 * Shape<T>::NB; }

// Leading dimension (in elements) of every coefficient block: widths are padded with
// zero columns to a multiple of 32 so that both element types see whole LDS stages.
constexpr int kLdAlign = 32;
inline int pad_ld(int d) { return (d + kLdAlign - 1) / kLdAlign * kLdAlign; }

constexpr int kMaxRowBlocks = 16;  // 16-row MFMA blocks per tile => at most 256 rows per tile

template <typename T> struct LayerArgs {
  const T *Hin;      // [n_points * rho][ldin] coefficient block entering the layer
  const T *W;        // [n_col_tiles * tile_cols][ldin] zero-padded weights
  const T *bias;     // [n_col_tiles * tile_cols] zero-padded bias
  const void *Whi;   // bf16 kernels only: hi and lo parts of W, [n_col_tiles * 128][ldin] bf16 each
  const void *Wlo;
  T *Hout;           // [n_points * out_rows][ldout]
  long n_points;
  long n_row_tiles;  // ceil(n_points / P)
  int n_col_tiles;
  int rho;           // coefficient rows per point
  int P;             // points per tile, P * rho <= 16 * MB
  int ldin;
  int ldout;
  int order;         // 2 or 4
  int R;             // directions in this pass
  int last;          // emit only the 0-th and the highest-order row(s)
  int act;           // 0 tanh, 1 identity, 2 sin
  int standard;      // 1: un-collapsed Taylor mode (1 + K*R rows per point), for comparison
  int out_rows;      // rows per point in Hout: rho, or when last: 2 (collapsed) / 1 + R (standard)
  T *Zout;           // forward that records a tape: the pre-activation rows [n_points * rho][ldout] go here too (else nullptr)
  const T *Zsaved;   // bwd == 1: recorded pre-activations of the layer whose rule is reversed, [n_points * rho][ldout]
  int bwd;           // 1: Hin holds cotangents, W the transposed weights, and the epilogue is the reverse of the
                     //    collapsed rule of that order (writes the cotangents of the pre-activations)
  int wpp = 1;  // wavefronts sharing one point in the rule: 4 / P for tiles of 1 or 2 points (forward, collapsed), else 1
  // plain-bf16 kernel only: Hin is a bf16 plane [rows][ldin]; out_bf16 != 0: Hout is one too (0: rows of T, the
  // last hidden layer's output for the final kernel)
  int out_bf16 = 0;
};

// Launch the stacked GEMM + fused jet rule for one layer.  MB in {4, 8, 9, 12, 13, 16}.
template <typename T> hipError_t launch_layer(const LayerArgs<T> &a, int MB, hipStream_t s);
bool row_blocks_supported(int MB);
// fp32 storage, bf16 matrix cores: nsplit = 3 (hi*hi + hi*lo + lo*hi) or 1 (hi*hi only)
hipError_t launch_layer_bf16(const LayerArgs<float> &a, int MB, int nsplit, hipStream_t s);
hipError_t launch_pack_bf16(const float *W, int d_out, int d_in, void *hi, void *lo, int rows_pad, int ld, hipStream_t s);
// Plain bf16 with 256-column tiles (same tile heights and points per tile as launch_layer_bf16): a.n_col_tiles counts
// 256-column tiles and Whi must be padded to that many rows.  Collapsed forward only.
constexpr int kWideCols = 256;
bool bf16_t256_supported(int MB, int wpp);
hipError_t launch_layer_bf16_t256(const LayerArgs<float> &a, int MB, hipStream_t s);

template <typename T> struct SeedArgs {
  const T *x;   // [N][D]
  const T *V;   // directions or nullptr (standard basis)
  T *out;       // [N * rho][ld]
  long N;
  long v_sn;    // element strides of V: point, direction, coordinate
  long v_sr;
  long v_sd;
  int D, ld, rho, order;
  int r0;       // index of this pass's first direction
  int standard; // row layout of un-collapsed Taylor mode
  int R;        // directions in this pass
  int out_bf16 = 0;  // 0: rows of T; 1: the block is written as bf16 (same [rows][ld] indexing)
};
template <typename T> hipError_t launch_seed(const SeedArgs<T> &a, hipStream_t s);

// First layer when every point shares the directions: no GEMM over the per-direction rows.
template <typename T> struct FirstArgs {
  const T *x;     // [N][D]
  const T *V;     // directions (element (n, r, k) at V[n*v_sn + r*v_sr + k*v_sd]) or nullptr (basis)
  const T *W;     // zero-padded first-layer weights [rows_pad][ld0]
  const T *WT;    // the same transposed, [ld0][ld1] (shared-direction kernels: consecutive features are consecutive words)
  const T *bias;  // [rows_pad]
  T *Z1;          // scratch [R][ld1]: W_1 v_r
  T *out;         // last == 0: [N * rho][ld1]; last == 1: [N][2][ld1]
  long N;
  long v_sr, v_sd;
  long v_sn = 0;  // point stride of V (0: shared by all points)
  int D, ld0, ld1, rho, order, R, r0, last, act;
  int standard;   // un-collapsed row layout
  int out_rows;   // rows per point in out
  int out_bf16 = 0;      // 0: rows of T; 1: out is written as bf16 (same indexing)
  long out_point0 = 0;   // index of this launch's first point in out (x and N are already offset)
  int cus = 256;         // compute units of the device (launch shape of small batches)
};
constexpr int kMaxOutputs = 1024;  // widest last layer (outputs are produced by a per-point dot-product kernel)
// 0: none (seed block + stacked GEMM); 1: directions shared by all points; 2: per-point directions with D <= 16
int first_layer_fast_path(int D, long v_point_stride, int R);
template <typename T> hipError_t launch_first(const FirstArgs<T> &a, hipStream_t s);

// transpose == 0: Wp[j][k] = W[j][k] (W is [d_out][d_in]); transpose == 1: Wp[j][k] = W[k][j] (W is [d_in][d_out]).
// bp may be nullptr.
template <typename T>
hipError_t launch_pack(const T *W, const T *b, int d_out, int d_in, T *Wp, T *bp, int rows_pad,
                       int ld, hipStream_t s, int transpose = 0);

// ---- reverse pass (collapsed, orders 2 and 4) -----------------------------------------------------
template <typename T> struct BwdLastArgs {
  const T *Z;     // recorded pre-activations of the last hidden layer [N * rho][ld]
  const T *w;     // last-layer weights [C][ld]
  const T *gu;    // dL/du [N][C] or nullptr
  const T *gop;   // dL/dop [N][C] or nullptr
  T *Zbar;        // out: cotangents of those pre-activations [N * rho][ld]
  long N;
  int ld, rho, R, act;
  int C;          // network outputs
  int order;      // 2 or 4
  double scale;
};
template <typename T> hipError_t launch_bwd_last(const BwdLastArgs<T> &a, hipStream_t s);

// For every output c < C: gw[c][j] = sum_n gu[n][c] pair[n][0][j] + scale gop[n][c] pair[n][1][j] (j < d, gw row pitch d),
// gbias[c] = sum_n gu[n][c]; scratch >= 65 * ld elements (reused output after output, in stream order)
template <typename T>
hipError_t launch_last_grads(const T *pair, const T *gu, const T *gop, double scale, long N, int ld, int d, int C, T *gw, T *gbias,
                             T *scratch, hipStream_t s, int accumulate = 0);
// gb[j] = sum_n Zbar[n * rho][j] (j < d); scratch >= 64 * ld elements
template <typename T>
hipError_t launch_bias_grad(const T *Zbar, long N, int rho, int ld, int d, T *gb, T *scratch, hipStream_t s, int accumulate = 0);
// gW[i][j] = sum_m Zbar[m][i] * H[m][j], i < d_out, j < d_in (gW row-major [d_out][d_in]); split over row ranges,
// partial sums in `partials` (wgrad_partial_elems elements), added in a fixed order; accumulate != 0 in these three
// launchers: add to what the output holds instead of overwriting it
size_t wgrad_partial_elems(long M, int d_out, int d_in);
template <typename T>
hipError_t launch_wgrad(const T *Zbar, int ld_out, const T *H, int ld_in, long M, int d_out, int d_in, T *gW, T *partials,
                        hipStream_t s, int accumulate = 0);

// Direction families of the exact biharmonic (interpolation with 4-jets): family 0: 4 e_d (D rows);
// family 1: 3 e_d1 + e_d2, d1 != d2 (D(D-1) rows); family 2: 2 e_d1 + 2 e_d2, d1 < d2 (D(D-1)/2 rows).
template <typename T> hipError_t launch_biharm_dirs(T *V, int D, int family, hipStream_t s);

// out[n][s][:] = sigma_n v_{n,s}; sigma_n = sigma + n*sig_stride ([D][K]), v_{n,s} = V + n*v_stride + s*K; Nd = N or 1
template <typename T>
hipError_t launch_sigma_dirs(const T *sigma, long sig_stride, const T *V, long v_stride, T *out, long Nd, int S, int D, int K,
                             hipStream_t s);

// One-workgroup path for tiny calls (ctm_small.hip): the whole call in one launch, coefficients resident in LDS.
constexpr int kSmallMaxLayers = 8;            // linear layers
constexpr int kSmallMaxRows = 256;            // N * rho
constexpr size_t kSmallMaxLds = 64 * 1024;    // two coefficient blocks + all weights
constexpr long kSmallMaxMacs = 1L << 20;      // multiply-adds of all hidden layers together
template <typename T> struct SmallArgs {
  const T *x;                      // [N][D]
  const T *V;                      // directions (element (n, r, k) at V[n*v_sn + r*v_sr + k*v_sd]) or nullptr (basis)
  long v_sn, v_sr, v_sd;
  const T *W[kSmallMaxLayers];     // packed weights of the handle: hidden layers zero-padded [>= ld[l+1]][ld[l]], last [C][ld[L-1]]
  const T *b[kSmallMaxLayers];     // padded biases; last: [C]
  int dims[kSmallMaxLayers + 1];
  int ld[kSmallMaxLayers];         // padded width of dims[l]
  int L, N, R, rho, order, act, C;
  int pitch;                       // LDS row pitch of the coefficient blocks (small_call_pitch)
  int accumulate;                  // 1: op += (u untouched), as in FinalArgs
  double scale;
  T *u, *op;                       // [N][C], may be nullptr
};
int small_call_pitch(const int *dims, int L);
size_t small_call_lds_bytes(const int *dims, int L, long rows, size_t elem_size);
template <typename T> hipError_t launch_small_call(const SmallArgs<T> &a, size_t lds_bytes, hipStream_t s);

template <typename T> struct FinalArgs {
  const T *pair;  // [N][1 + nk][ld] : h_0 and the nk highest-order rows of the last hidden layer
  int nk;         // 1 (collapsed) or R (un-collapsed: summed here)
  const T *w;     // [C][ld] zero-padded last-layer weights
  const T *b;     // [C]
  T *u;           // [N][C], may be nullptr
  T *op;          // [N][C], may be nullptr
  long N;
  int ld;
  int C;          // network outputs
  double scale;
  int accumulate;  // 0: write u and op; 1: op += (later passes over a split direction set)
};
template <typename T> hipError_t launch_final(const FinalArgs<T> &a, hipStream_t s);

}  // namespace ctm
