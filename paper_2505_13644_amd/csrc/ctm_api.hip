// C ABI of libctm.so: argument validation, tiling plan, workspace carving and the
// per-call launch sequence  seed -> (stacked GEMM + jet rule) per hidden layer -> last layer.
#include <atomic>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <mutex>
#include <new>
#include <string>
#include <type_traits>
#include <unordered_map>
#include <vector>

#include "../../include/ctm.h"
#include "../../include/ctm_bench.h"
#include "ctm_internal.h"

using namespace ctm;

// Device memory of ctm_laplacian_static: one array per GPU the library runs on, held until the process ends.
// In host code the name is only a handle for hipGetSymbolAddress; kernels and copies get the address it returns.
static __device__ __align__(256) unsigned char scratch[CTM_STATIC_SCRATCH_BYTES];

namespace {

thread_local std::string g_err;

int fail(int code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

int fail_hip(hipError_t e, const char *what) {
  return fail(CTM_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

size_t elem_size(ctm_dtype t) { return t == CTM_F64 ? 8 : 4; }
size_t round256(size_t b) { return (b + 255) / 256 * 256; }

struct PassPlan {
  int R, rho, MB, P;
};

// Optional per-kernel timing for benchmarks (ctm_profile_begin / ctm_profile_end).
struct Profile {
  bool on = false;
  std::vector<hipEvent_t> ev;  // ev[i], ev[i+1] bracket interval i
  std::vector<int> cls;        // kernel class of interval i, or -1 for a gap between calls
};
thread_local Profile g_prof;

hipError_t prof_mark(hipStream_t st, int cls_of_preceding) {
  if (!g_prof.on) return hipSuccess;
  hipEvent_t e;
  hipError_t rc = hipEventCreate(&e);
  if (rc != hipSuccess) return rc;
  rc = hipEventRecord(e, st);
  if (rc != hipSuccess) { (void)hipEventDestroy(e); return rc; }
  if (!g_prof.ev.empty()) g_prof.cls.push_back(cls_of_preceding);
  g_prof.ev.push_back(e);
  return hipSuccess;
}

// collapsed: 1 + (K-1) R + 1 rows; un-collapsed ("standard"): 1 + K R rows (Sec. 3.1)
long rows_per_point(int K, int R, bool standard = false) {
  return standard ? 1L + (long)K * R : 1L + (long)(K - 1) * R + 1L;
}

// Largest direction count whose rows fit one tile of kMaxRowBlocks MFMA row blocks.
int max_dirs_per_pass(int K, bool standard = false) {
  return standard ? (16 * kMaxRowBlocks - 1) / K : (16 * kMaxRowBlocks - 2) / (K - 1);
}

// Pick the row-block count that wastes the fewest MFMA rows (ties: the taller tile).  When that tile
// shape leaves the GPU under-filled (fewer than `slots` tiles, i.e. fewer than two per compute unit: small
// batches), fall back to the shortest tile whose row efficiency is within 7 % of the best and that reaches
// `slots` tiles, or to the shortest such tile if none does.  col_tiles = column tiles of the narrowest layer
// (one tile shape per pass).
PassPlan plan_pass(int K, int R, bool standard = false, long N = -1, int col_tiles = 1, int slots = 512) {
  PassPlan best{R, (int)rows_per_point(K, R, standard), 0, 0};
  double best_eff = -1.0;
  static const int kChoices[] = {4, 8, 9, 12, 13, 16};
  for (int MB : kChoices) {  // ascending, so a tie goes to the taller tile
    const int P = 16 * MB / best.rho;
    if (P < 1) continue;
    const double eff = (double)P * best.rho / (16.0 * MB);
    if (eff >= best_eff - 1e-12) {
      best.MB = MB;
      best.P = P;
      if (eff > best_eff) best_eff = eff;
    }
  }
  if (N < 0) return best;
  auto tiles_of = [&](int P) { return ((N + P - 1) / P) * (long)col_tiles; };
  if (tiles_of(best.P) >= slots) return best;
  PassPlan small = best;
  bool have = false;
  for (int MB : kChoices) {
    const int P = 16 * MB / best.rho;
    if (P < 1 || MB >= best.MB) continue;
    const double eff = (double)P * best.rho / (16.0 * MB);
    if (eff < best_eff - 0.07) continue;
    if (!have) {  // shortest admissible tile
      small.MB = MB;
      small.P = P;
      have = true;
      if (tiles_of(P) < slots) return small;  // even the shortest does not fill the slots: take it
    }
    if (tiles_of(P) >= slots) {  // keep growing while the slots stay filled
      small.MB = MB;
      small.P = P;
    }
  }
  return small;
}

// ---- interpolation coefficients gamma_{i,j} (App. E, general coefficient formula for gamma_{i,j}), exact rational arithmetic
struct Frac {
  long long n = 0, d = 1;
};
long long gcd_ll(long long a, long long b) {
  a = a < 0 ? -a : a;
  b = b < 0 ? -b : b;
  while (b) { long long t = a % b; a = b; b = t; }
  return a ? a : 1;
}
Frac norm(Frac f) {
  if (f.d < 0) { f.n = -f.n; f.d = -f.d; }
  const long long g = gcd_ll(f.n, f.d);
  f.n /= g; f.d /= g;
  return f;
}
// Products are formed in 128 bits and reduced before they return to 64: the intermediates of the coefficient formula
// at |i| = 8 pass 1e17, and a product of two of those would not fit.  `overflow` is raised if a reduced value still
// does not fit 63 bits (none does for |i| <= 8, I <= 4; checked against exact big-integer fractions in the tests).
thread_local bool g_frac_overflow = false;
__int128 gcd128(__int128 a, __int128 b) {
  a = a < 0 ? -a : a;
  b = b < 0 ? -b : b;
  while (b) { __int128 t = a % b; a = b; b = t; }
  return a ? a : 1;
}
Frac reduce128(__int128 n, __int128 d) {
  if (d < 0) { n = -n; d = -d; }
  const __int128 g = gcd128(n, d);
  n /= g; d /= g;
  const __int128 lim = (__int128)0x7fffffffffffffffLL;
  if (n > lim || n < -lim || d > lim) g_frac_overflow = true;
  return Frac{(long long)n, (long long)d};
}
Frac mul(Frac a, Frac b) { return reduce128((__int128)a.n * b.n, (__int128)a.d * b.d); }
Frac add(Frac a, Frac b) {
  const long long g = gcd_ll(a.d, b.d);   // common denominator lcm(a.d, b.d), not a.d * b.d
  return reduce128((__int128)a.n * (b.d / g) + (__int128)b.n * (a.d / g), (__int128)a.d * (b.d / g));
}
// generalised binomial (a over b) = prod_{l<b} (a - l) / (b - l), a rational, b a non-negative integer
Frac gbinom(Frac a, int b) {
  Frac r{1, 1};
  for (int l = 0; l < b; ++l) r = mul(r, norm(Frac{a.n - (long long)l * a.d, a.d * (long long)(b - l)}));
  return r;
}
// gamma_{i,j} = sum_{0 < m <= i} (-1)^{|i-m|} (i over m) (|i| m/|m| over j) (|m|/|i|)^{|i|}
Frac interp_gamma(int I, const int *iv, const int *jv) {
  int isum = 0;
  for (int t = 0; t < I; ++t) isum += iv[t];
  Frac total{0, 1};
  std::vector<int> m(I, 0);
  while (true) {
    int t = 0;  // next multi-index m in the box [0, i]
    while (t < I && m[t] == iv[t]) m[t++] = 0;
    if (t == I) break;
    ++m[t];
    int msum = 0, dist = 0;
    for (int q = 0; q < I; ++q) { msum += m[q]; dist += iv[q] - m[q]; }
    Frac term{(dist & 1) ? -1 : 1, 1};
    for (int q = 0; q < I; ++q) {
      term = mul(term, gbinom(Frac{iv[q], 1}, m[q]));
      term = mul(term, gbinom(norm(Frac{(long long)isum * m[q], msum}), jv[q]));
    }
    for (int q = 0; q < isum; ++q) term = mul(term, norm(Frac{msum, isum}));
    total = add(total, term);
  }
  return total;
}

struct Split {
  int n_passes, first, lastR;  // passes 0..n-2 take `first` directions, the last one `lastR`
};
Split split_dirs(int K, int R, bool standard = false) {
  const int cap = max_dirs_per_pass(K, standard);
  Split s;
  s.n_passes = (R + cap - 1) / cap;
  s.first = (R + s.n_passes - 1) / s.n_passes;
  s.lastR = R - (s.n_passes - 1) * s.first;
  return s;
}

}  // namespace

struct ctm_mlp {
  int L = 0;                 // linear layers
  std::vector<int> dims;     // L + 1
  std::vector<int> ld;       // padded widths of dims[0..L-1]
  std::vector<int> col_tiles;  // per hidden layer l = 0..L-2
  ctm_dtype dtype = CTM_F32;
  ctm_act act = CTM_ACT_TANH;
  int device = 0;
  void *arena = nullptr;
  std::vector<void *> Wp, bp;  // l < L-1: padded matrices; l = L-1: [dims[L]][ld] and [dims[L]]
  std::vector<void *> Whi, Wlo;  // bf16 variants: split weights of the hidden layers
  int cus = 256;                 // compute units of the handle's device
  int slots = 512;               // under-fill threshold of the tile plan: two tiles per compute unit.  Deliberately below the 3-4
                                 // workgroups a CU can hold: with 2-3 tiles per CU the most row-efficient tile still measured
                                 // faster than a shorter one (weighted Laplacian, N = 2048: 5-25 % slower with shorter tiles)
  int min_col_tiles = 1;         // fewest column tiles among the hidden layers
  std::vector<void *> WT;        // l = 1..L-2: W_l transposed, [pad(dims[l])][ld(dims[l+1])], for the reverse pass
  void *W1T = nullptr;           // W_1 transposed, [ld(dims[0])][ld(dims[1])], for the shared-direction first-layer kernels
  // The reverse pass reads the weights from the handle, so it must find the weights its forward ran with: every
  // ctm_update_mlp bumps `version`, a recording forward notes the version under its tape's address, and the matching
  // reverse pass refuses to run on another version.  (Bounded: the notes are dropped once there are kMaxTapeNotes.)
  static constexpr size_t kMaxTapeNotes = 1024;
  mutable std::mutex mu;
  unsigned long long version = 1;
  mutable std::unordered_map<const void *, unsigned long long> tape_version;
  void note_tape(const void *tape) const {
    std::lock_guard<std::mutex> g(mu);
    if (tape_version.size() >= kMaxTapeNotes) tape_version.clear();
    tape_version[tape] = version;
  }
  // true unless the tape is known to come from a forward with other weights than the handle holds now
  bool tape_matches(const void *tape) const {
    std::lock_guard<std::mutex> g(mu);
    auto it = tape_version.find(tape);
    return it == tape_version.end() || it->second == version;
  }
};

namespace {

int tile_cols_of(ctm_dtype t) { return t == CTM_F64 ? tile_cols<double>() : tile_cols<float>(); }
bool is_bf16(ctm_dtype t) { return t == CTM_F32_BF16X3 || t == CTM_F32_BF16; }
bool known_dtype(ctm_dtype t) { return t == CTM_F64 || t == CTM_F32 || is_bf16(t); }

struct Layout {
  size_t block_bytes, pair_bytes, dirs_bytes, total;
};
Layout workspace_layout(const ctm_mlp *m, int K, long N, int Rpass, bool standard = false) {
  const size_t es = elem_size(m->dtype);
  int maxld = 0;
  for (int l = 0; l + 1 < m->L; ++l) maxld = m->ld[l] > maxld ? m->ld[l] : maxld;  // inputs of hidden layers
  Layout lo;
  lo.block_bytes = round256((size_t)N * (size_t)rows_per_point(K, Rpass, standard) * (size_t)maxld * es);
  lo.pair_bytes = round256((size_t)N * (standard ? 1 + (size_t)Rpass : 2) * (size_t)m->ld[m->L - 1] * es);
  lo.dirs_bytes = round256((size_t)Rpass * (size_t)m->ld[1] * es);  // W_1 v_r rows
  lo.total = 2 * lo.block_bytes + lo.pair_bytes + lo.dirs_bytes;
  return lo;
}

// Calls small enough for the one-launch path: all coefficient rows in one workgroup, blocks and one weight matrix in
// LDS, a bounded amount of arithmetic, storage-type arithmetic (not the bf16 variants), collapsed mode.
bool small_call_fits(const ctm_mlp *m, int K, long N, int R) {
  if (is_bf16(m->dtype) || m->L > kSmallMaxLayers) return false;
  const long rho = rows_per_point(K, R);
  if (N > kSmallMaxRows || N * rho > kSmallMaxRows) return false;
  if (small_call_lds_bytes(m->dims.data(), m->L, N * rho, elem_size(m->dtype)) > kSmallMaxLds) return false;
  long macs = 0;
  for (int l = 0; l + 1 < m->L; ++l) macs += N * rho * (long)m->dims[l] * m->dims[l + 1];
  return macs <= kSmallMaxMacs;
}

template <typename T>
int run_small(const ctm_mlp *m, int K, const T *x, long N, const T *V, int R, long sn, long sr, long sd, double scale, T *u, T *op,
              hipStream_t st, bool accumulate) {
  SmallArgs<T> a = {};
  a.x = x; a.V = V; a.v_sn = sn; a.v_sr = sr; a.v_sd = sd;
  a.L = m->L; a.N = (int)N; a.R = R; a.rho = (int)rows_per_point(K, R); a.order = K; a.act = (int)m->act; a.C = m->dims[m->L];
  a.accumulate = accumulate ? 1 : 0; a.scale = scale; a.u = u; a.op = op;
  for (int l = 0; l < m->L; ++l) {
    a.W[l] = (const T *)m->Wp[l]; a.b[l] = (const T *)m->bp[l]; a.ld[l] = m->ld[l];
  }
  a.pitch = small_call_pitch(m->dims.data(), m->L);
  for (int l = 0; l <= m->L; ++l) a.dims[l] = m->dims[l];
  if (prof_mark(st, -1) != hipSuccess) return fail(CTM_ERR_HIP, "profiling event failed");
  hipError_t e = launch_small_call<T>(a, small_call_lds_bytes(m->dims.data(), m->L, N * a.rho, sizeof(T)), st);
  if (e != hipSuccess) return fail_hip(e, "one-launch kernel");
  (void)prof_mark(st, 1);
  return CTM_OK;
}

template <typename T>
int run_passes(const ctm_mlp *m, int K, const T *x, long N, const T *V, int R, long sn, long sr, long sd,
               double scale, T *u, T *op, void *ws, hipStream_t st, bool accumulate_first = false,
               bool standard = false) {
  if (!standard && small_call_fits(m, K, N, R)) return run_small<T>(m, K, x, N, V, R, sn, sr, sd, scale, u, op, st, accumulate_first);
  const Split sp = split_dirs(K, R, standard);
  const Layout lo = workspace_layout(m, K, N, sp.first, standard);
  T *buf[2] = {reinterpret_cast<T *>(ws), reinterpret_cast<T *>((char *)ws + lo.block_bytes)};
  T *pair = reinterpret_cast<T *>((char *)ws + 2 * lo.block_bytes);
  T *dirs = reinterpret_cast<T *>((char *)ws + 2 * lo.block_bytes + lo.pair_bytes);
  const int L = m->L;
  if (prof_mark(st, -1) != hipSuccess) return fail(CTM_ERR_HIP, "profiling event failed");
  for (int pass = 0; pass < sp.n_passes; ++pass) {
    const int Rp = (pass == sp.n_passes - 1) ? sp.lastR : sp.first;
    const PassPlan pl = plan_pass(K, Rp, standard, N, m->min_col_tiles, m->slots);
    const int last_rows = standard ? 1 + Rp : 2;
    const int fast_first = first_layer_fast_path(m->dims[0], sn, Rp);
    // plain-bf16 handles keep the blocks between layers as one bf16 plane; see ctm_layer_bf16.hip
    const int bf16_blocks = m->dtype == CTM_F32_BF16 ? 1 : 0;
    const T *in = buf[1];
    int l_begin = 0;
    hipError_t e;
    if (fast_first) {
      // shared directions: the first layer is written directly, without a seed block or a GEMM
      const bool last = (L == 2);
      FirstArgs<T> fa;
      fa.x = x; fa.V = V; fa.W = (const T *)m->Wp[0]; fa.WT = (const T *)m->W1T; fa.bias = (const T *)m->bp[0]; fa.cus = m->cus;
      fa.Z1 = dirs;
      fa.out = last ? pair : buf[0];
      fa.N = N; fa.v_sn = sn; fa.v_sr = sr; fa.v_sd = sd;
      fa.D = m->dims[0]; fa.ld0 = m->ld[0]; fa.ld1 = m->ld[1]; fa.rho = pl.rho; fa.order = K; fa.R = Rp;
      fa.r0 = pass * sp.first; fa.last = last ? 1 : 0; fa.act = (int)m->act;
      fa.standard = standard ? 1 : 0; fa.out_rows = last ? last_rows : pl.rho;
      fa.out_bf16 = last ? 0 : bf16_blocks;
      e = launch_first<T>(fa, st);
      if (e != hipSuccess) return fail_hip(e, "first-layer kernel launch");
      (void)prof_mark(st, 0);
      in = fa.out;
      l_begin = 1;
    } else {
      SeedArgs<T> sa;
      sa.x = x; sa.V = V; sa.out = buf[1]; sa.N = N;
      sa.v_sn = sn; sa.v_sr = sr; sa.v_sd = sd;
      sa.D = m->dims[0]; sa.ld = m->ld[0]; sa.rho = pl.rho; sa.order = K; sa.r0 = pass * sp.first;
      sa.standard = standard ? 1 : 0; sa.R = Rp; sa.out_bf16 = bf16_blocks;
      e = launch_seed<T>(sa, st);
      if (e != hipSuccess) return fail_hip(e, "seed kernel launch");
      (void)prof_mark(st, 0);
    }
    for (int l = l_begin; l + 1 < L; ++l) {
      const bool last = (l == L - 2);
      T *out = last ? pair : buf[l & 1];
      LayerArgs<T> la;
      la.Hin = in; la.W = (const T *)m->Wp[l]; la.bias = (const T *)m->bp[l]; la.Hout = out;
      la.n_points = N; la.n_row_tiles = (N + pl.P - 1) / pl.P; la.n_col_tiles = m->col_tiles[l];
      la.rho = pl.rho; la.P = pl.P; la.ldin = m->ld[l]; la.ldout = m->ld[l + 1];
      la.order = K; la.R = Rp; la.last = last ? 1 : 0; la.act = (int)m->act;
      la.standard = standard ? 1 : 0; la.out_rows = last ? last_rows : pl.rho;
      la.Whi = nullptr; la.Wlo = nullptr; la.Zout = nullptr; la.Zsaved = nullptr; la.bwd = 0;
      la.wpp = (standard || pl.P > 2) ? 1 : 4 / pl.P;
      bool done = false;
      if constexpr (std::is_same<T, float>::value) {
        if (is_bf16(m->dtype)) {
          la.Whi = m->Whi[l]; la.Wlo = m->Wlo[l];
          la.out_bf16 = last ? 0 : bf16_blocks;
          // plain bf16: 256-column tiles where the layer is wide enough to fill them (at most a fifth of the columns of its
          // tiles padding) and the batch gives every compute unit at least two of them
          const long wide_ct = (m->ld[l + 1] + kWideCols - 1) / kWideCols;
          const bool wide = m->dtype == CTM_F32_BF16 && !standard && bf16_t256_supported(pl.MB, la.wpp) &&
                            5 * (long)m->ld[l + 1] >= 4 * wide_ct * kWideCols && la.n_row_tiles * wide_ct >= 2L * m->cus;
          if (wide) {
            la.n_col_tiles = (int)wide_ct;
            e = launch_layer_bf16_t256(la, pl.MB, st);
          } else {
            e = launch_layer_bf16(la, pl.MB, m->dtype == CTM_F32_BF16X3 ? 3 : 1, st);
          }
          done = true;
        }
      }
      if (!done) e = launch_layer<T>(la, pl.MB, st);
      if (e != hipSuccess) return fail_hip(e, "layer kernel launch");
      (void)prof_mark(st, 1);
      in = out;
    }
    FinalArgs<T> fa;
    fa.pair = pair; fa.nk = standard ? Rp : 1; fa.w = (const T *)m->Wp[L - 1]; fa.b = (const T *)m->bp[L - 1];
    fa.u = u; fa.op = op; fa.N = N; fa.ld = m->ld[L - 1]; fa.C = m->dims[L]; fa.scale = scale; fa.accumulate = (pass > 0 || accumulate_first) ? 1 : 0;
    e = launch_final<T>(fa, st);
    if (e != hipSuccess) return fail_hip(e, "final kernel launch");
    (void)prof_mark(st, 2);
  }
  return CTM_OK;
}

}  // namespace
extern "C" size_t ctm_workspace_bytes_standard(const ctm_mlp *m, int K, long N, int R);
namespace {
bool misaligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) != 0; }

// The handle's weights live on the device that was current at ctm_create_mlp; calls must be made with it current.
int check_device(const ctm_mlp *m, const char *who) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
  if (dev != m->device)
    return fail(CTM_ERR_UNSUPPORTED, "%s: the handle belongs to device %d but device %d is current", who, m->device, dev);
  return CTM_OK;
}

// Address of the current device's copy of `scratch`: looked up once per device, with that device current
// (every GPU holds its own copy of the array at its own address).
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];
int static_scratch(int device, const char *who, void **out) {
  if (device < 0 || device >= kMaxDevices) return fail(CTM_ERR_UNSUPPORTED, "%s: device index %d is out of range", who, device);
  void *p = g_scratch_ptr[device].load(std::memory_order_acquire);
  if (!p) {
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return fail_hip(e, "hipGetSymbolAddress of the built-in scratch array");
    if (!p) return fail(CTM_ERR_HIP, "%s: the built-in scratch array has no device address", who);
    g_scratch_ptr[device].store(p, std::memory_order_release);
  }
  *out = p;
  return CTM_OK;
}

int run_operator(const ctm_mlp *m, int K, const void *x, long N, const void *V, int R, long sn, long sr,
                 long sd, double scale, void *u, void *op, void *ws, size_t ws_bytes, void *stream,
                 const char *who, bool standard = false) {
  if (!m) return fail(CTM_ERR_NULL, "%s: mlp handle is NULL", who);
  if (!x) return fail(CTM_ERR_NULL, "%s: x is NULL", who);
  if (N < 1) return fail(CTM_ERR_SHAPE, "%s: N = %ld, need N >= 1", who, N);
  if (R < 1) return fail(CTM_ERR_SHAPE, "%s: %d directions, need at least 1", who, R);
  if (N > (1L << 40) / rows_per_point(K, R, standard)) return fail(CTM_ERR_SHAPE, "%s: N * rows per point overflows", who);
  if (!ws) return fail(CTM_ERR_NULL, "%s: workspace is NULL", who);
  const size_t need = standard ? ctm_workspace_bytes_standard(m, K, N, R) : ctm_workspace_bytes(m, K, N, R);
  if (ws_bytes < need)
    return fail(CTM_ERR_WORKSPACE, "%s: workspace has %zu bytes, need %zu", who, ws_bytes, need);
  const size_t es = elem_size(m->dtype);
  if (misaligned(ws, 256)) return fail(CTM_ERR_ALIGN, "%s: workspace must be 256-byte aligned", who);
  if (misaligned(x, es) || misaligned(V, es) || misaligned(u, es) || misaligned(op, es))
    return fail(CTM_ERR_ALIGN, "%s: x, directions, u and op must be aligned to the element size", who);
  if (int rc = check_device(m, who)) return rc;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (m->dtype == CTM_F64)
    return run_passes<double>(m, K, (const double *)x, N, (const double *)V, R, sn, sr, sd, scale, (double *)u,
                              (double *)op, ws, st, false, standard);
  return run_passes<float>(m, K, (const float *)x, N, (const float *)V, R, sn, sr, sd, scale, (float *)u,
                           (float *)op, ws, st, false, standard);
}

template <typename T> hipError_t pack_all(ctm_mlp *m, const void *const *W, const void *const *b, hipStream_t st) {
  for (int l = 0; l < m->L; ++l) {
    const bool lastl = (l == m->L - 1);
    const int rows_pad = lastl ? m->dims[m->L] : m->col_tiles[l] * tile_cols<T>();
    const T *bl = (b && b[l]) ? (const T *)b[l] : nullptr;
    hipError_t e = launch_pack<T>((const T *)W[l], bl, m->dims[l + 1], m->dims[l], (T *)m->Wp[l], (T *)m->bp[l],
                                  rows_pad, m->ld[l], st);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t pack_everything(ctm_mlp *m, const void *const *W, const void *const *b, hipStream_t st) {
  hipError_t e = (m->dtype == CTM_F64) ? pack_all<double>(m, W, b, st) : pack_all<float>(m, W, b, st);
  const int bn = tile_cols_of(m->dtype);
  for (int l = 0; e == hipSuccess && is_bf16(m->dtype) && l + 1 < m->L; ++l)
    e = launch_pack_bf16((const float *)W[l], m->dims[l + 1], m->dims[l], m->Whi[l], m->Wlo[l],
                         (m->col_tiles[l] * bn + kWideCols - 1) / kWideCols * kWideCols, m->ld[l], st);
  if (e == hipSuccess && m->L >= 2) {
    if (m->dtype == CTM_F64)
      e = launch_pack<double>((const double *)W[0], nullptr, m->dims[0], m->dims[1], (double *)m->W1T, nullptr, m->ld[0], m->ld[1], st, 1);
    else
      e = launch_pack<float>((const float *)W[0], nullptr, m->dims[0], m->dims[1], (float *)m->W1T, nullptr, m->ld[0], m->ld[1], st, 1);
  }
  for (int l = 1; e == hipSuccess && l + 1 < m->L; ++l) {
    const int rows_pad = m->col_tiles[l - 1] * bn;
    if (m->dtype == CTM_F64)
      e = launch_pack<double>((const double *)W[l], nullptr, m->dims[l], m->dims[l + 1], (double *)m->WT[l], nullptr, rows_pad,
                              m->ld[l + 1], st, 1);
    else
      e = launch_pack<float>((const float *)W[l], nullptr, m->dims[l], m->dims[l + 1], (float *)m->WT[l], nullptr, rows_pad,
                             m->ld[l + 1], st, 1);
  }
  return e;
}

// ---- tape of a recording forward pass (collapsed, order K, one pass) ---------------------------------
struct TapeLayout {
  size_t h0;                  // seed block [M][ld0]
  std::vector<size_t> z, h;   // per hidden layer i (width dims[i+1]): pre-activations; outputs (all but the last hidden layer)
  size_t pair, total;
};
TapeLayout tape_layout(const ctm_mlp *m, int K, long N, int R) {
  const size_t es = elem_size(m->dtype);
  const size_t M = (size_t)N * (size_t)rows_per_point(K, R);
  TapeLayout t;
  size_t off = 0;
  t.h0 = off;
  off += round256(M * m->ld[0] * es);
  for (int i = 0; i + 1 < m->L; ++i) {
    t.z.push_back(off);
    off += round256(M * m->ld[i + 1] * es);
    t.h.push_back(off);
    if (i + 2 < m->L) off += round256(M * m->ld[i + 1] * es);
  }
  t.pair = off;
  off += round256((size_t)N * 2 * m->ld[m->L - 1] * es);
  t.total = off;
  return t;
}

struct BwdLayout {
  size_t block_bytes, scratch, partials, total;
};
BwdLayout bwd_layout(const ctm_mlp *m, int K, long N, int R) {
  const size_t es = elem_size(m->dtype);
  const long M = N * rows_per_point(K, R);
  int maxld = 0;
  size_t maxpart = 0;
  for (int i = 0; i + 1 < m->L; ++i) {
    maxld = m->ld[i + 1] > maxld ? m->ld[i + 1] : maxld;
    const size_t pe = wgrad_partial_elems(M, m->dims[i + 1], m->dims[i]);
    maxpart = pe > maxpart ? pe : maxpart;
  }
  BwdLayout b;
  b.block_bytes = round256((size_t)M * maxld * es);
  b.scratch = 2 * b.block_bytes;
  b.partials = b.scratch + round256(((size_t)(65 + m->dims[m->L]) * maxld + m->dims[m->L] + 64) * es);
  b.total = b.partials + round256(maxpart * es);
  return b;
}

int check_tape_call(const ctm_mlp *m, int K, long N, int R, const char *who) {
  if (!m) return fail(CTM_ERR_NULL, "%s: mlp handle is NULL", who);
  if (m->dtype != CTM_F64 && m->dtype != CTM_F32)
    return fail(CTM_ERR_UNSUPPORTED, "%s: the recording forward and the reverse pass are built for CTM_F32 and CTM_F64", who);
  if (N < 1) return fail(CTM_ERR_SHAPE, "%s: N = %ld, need N >= 1", who, N);
  if (R < 1) return fail(CTM_ERR_SHAPE, "%s: %d directions, need at least 1", who, R);
  if (N > (1L << 40) / rows_per_point(K, R)) return fail(CTM_ERR_SHAPE, "%s: N * rows per point overflows", who);
  return CTM_OK;
}

template <typename T>
int run_fwd_tape(const ctm_mlp *m, int K, const T *x, long N, const T *V, int R, long sn, double scale, T *u, T *op, void *tape,
                 hipStream_t st, bool accumulate_op = false, int r0 = 0) {
  const TapeLayout tl = tape_layout(m, K, N, R);
  const PassPlan pl = plan_pass(K, R, false, N, m->min_col_tiles, m->slots);
  const int L = m->L;
  char *tp = (char *)tape;
  SeedArgs<T> sa;
  sa.x = x; sa.V = V; sa.out = (T *)(tp + tl.h0); sa.N = N;
  sa.v_sn = sn; sa.v_sr = m->dims[0]; sa.v_sd = 1;
  sa.D = m->dims[0]; sa.ld = m->ld[0]; sa.rho = pl.rho; sa.order = K; sa.r0 = r0; sa.standard = 0; sa.R = R;
  if (prof_mark(st, -1) != hipSuccess) return fail(CTM_ERR_HIP, "profiling event failed");
  hipError_t e = launch_seed<T>(sa, st);
  if (e != hipSuccess) return fail_hip(e, "seed kernel launch");
  (void)prof_mark(st, 0);
  const T *in = sa.out;
  T *pair = (T *)(tp + tl.pair);
  for (int i = 0; i + 1 < L; ++i) {
    const bool last = (i == L - 2);
    LayerArgs<T> la;
    la.Hin = in; la.W = (const T *)m->Wp[i]; la.bias = (const T *)m->bp[i]; la.Whi = nullptr; la.Wlo = nullptr;
    la.Hout = last ? pair : (T *)(tp + tl.h[i]);
    la.n_points = N; la.n_row_tiles = (N + pl.P - 1) / pl.P; la.n_col_tiles = m->col_tiles[i];
    la.rho = pl.rho; la.P = pl.P; la.ldin = m->ld[i]; la.ldout = m->ld[i + 1];
    la.order = K; la.R = R; la.last = last ? 1 : 0; la.act = (int)m->act; la.standard = 0;
    la.out_rows = last ? 2 : pl.rho;
    la.Zout = (T *)(tp + tl.z[i]); la.Zsaved = nullptr; la.bwd = 0;
    la.wpp = pl.P > 2 ? 1 : 4 / pl.P;
    e = launch_layer<T>(la, pl.MB, st);
    if (e != hipSuccess) return fail_hip(e, "layer kernel launch");
    (void)prof_mark(st, 1);
    in = la.Hout;
  }
  FinalArgs<T> fa;
  fa.pair = pair; fa.nk = 1; fa.w = (const T *)m->Wp[L - 1]; fa.b = (const T *)m->bp[L - 1];
  fa.u = u; fa.op = op; fa.N = N; fa.ld = m->ld[L - 1]; fa.C = m->dims[L]; fa.scale = scale; fa.accumulate = accumulate_op ? 1 : 0;
  e = launch_final<T>(fa, st);
  if (e != hipSuccess) return fail_hip(e, "final kernel launch");
  (void)prof_mark(st, 2);
  return CTM_OK;
}

template <typename T>
int run_bwd(const ctm_mlp *m, int K, long N, int R, double scale, const void *tape, const T *gu, const T *gop, void *const *gW,
            void *const *gb, void *ws, hipStream_t st, int accumulate = 0) {
  const TapeLayout tl = tape_layout(m, K, N, R);
  const BwdLayout bl = bwd_layout(m, K, N, R);
  const PassPlan pl = plan_pass(K, R, false, N, m->min_col_tiles, m->slots);
  const int L = m->L;
  const long M = N * pl.rho;
  const char *tp = (const char *)tape;
  T *zb[2] = {(T *)ws, (T *)((char *)ws + bl.block_bytes)};
  T *scratch = (T *)((char *)ws + bl.scratch);
  T *partials = (T *)((char *)ws + bl.partials);
  int maxld = 0;
  for (int i = 0; i + 1 < L; ++i) maxld = m->ld[i + 1] > maxld ? m->ld[i + 1] : maxld;
  const int C = m->dims[L];
  T *dummy = scratch + 65 * (size_t)maxld;  // C * (maxld + 1) + 64 spare elements for gradients the caller does not want
  if (prof_mark(st, -1) != hipSuccess) return fail(CTM_ERR_HIP, "profiling event failed");

  int cur = 0;
  BwdLastArgs<T> ba;
  ba.Z = (const T *)(tp + tl.z[L - 2]); ba.w = (const T *)m->Wp[L - 1]; ba.gu = gu; ba.gop = gop; ba.Zbar = zb[cur];
  ba.N = N; ba.ld = m->ld[L - 1]; ba.rho = pl.rho; ba.R = R; ba.act = (int)m->act; ba.scale = scale; ba.C = m->dims[L]; ba.order = K;
  hipError_t e = launch_bwd_last<T>(ba, st);
  if (e != hipSuccess) return fail_hip(e, "reverse last-layer kernel launch");
  T *gw_last = (gW && gW[L - 1]) ? (T *)gW[L - 1] : dummy;
  T *gb_last = (gb && gb[L - 1]) ? (T *)gb[L - 1] : dummy + (size_t)C * maxld;
  e = launch_last_grads<T>((const T *)(tp + tl.pair), gu, gop, scale, N, m->ld[L - 1], m->dims[L - 1], C, gw_last, gb_last, scratch, st, accumulate);
  if (e != hipSuccess) return fail_hip(e, "last-layer gradient kernel launch");
  (void)prof_mark(st, 0);

  for (int i = L - 2; i >= 0; --i) {
    const T *Zb = zb[cur];
    if (gb && gb[i]) {
      e = launch_bias_grad<T>(Zb, N, pl.rho, m->ld[i + 1], m->dims[i + 1], (T *)gb[i], scratch, st, accumulate);
      if (e != hipSuccess) return fail_hip(e, "bias gradient kernel launch");
    }
    if (gW && gW[i]) {
      const T *Hprev = (const T *)(tp + (i == 0 ? tl.h0 : tl.h[i - 1]));
      e = launch_wgrad<T>(Zb, m->ld[i + 1], Hprev, m->ld[i], M, m->dims[i + 1], m->dims[i], (T *)gW[i], partials, st, accumulate);
      if (e != hipSuccess) return fail_hip(e, "weight gradient kernel launch");
    }
    (void)prof_mark(st, 2);
    if (i >= 1) {
      LayerArgs<T> la;
      la.Hin = Zb; la.W = (const T *)m->WT[i]; la.bias = (const T *)m->bp[i - 1]; la.Whi = nullptr; la.Wlo = nullptr;
      la.Hout = zb[cur ^ 1];
      la.n_points = N; la.n_row_tiles = (N + pl.P - 1) / pl.P; la.n_col_tiles = m->col_tiles[i - 1];
      la.rho = pl.rho; la.P = pl.P; la.ldin = m->ld[i + 1]; la.ldout = m->ld[i];
      la.order = K; la.R = R; la.last = 0; la.act = (int)m->act; la.standard = 0; la.out_rows = pl.rho;
      la.Zout = nullptr; la.Zsaved = (const T *)(tp + tl.z[i - 1]); la.bwd = 1;
      e = launch_layer<T>(la, pl.MB, st);
      if (e != hipSuccess) return fail_hip(e, "reverse layer kernel launch");
      (void)prof_mark(st, 1);
      cur ^= 1;
    }
  }
  return CTM_OK;
}

// ---- direction sets that need several passes (more rows per point than one tile holds) ----------------------------
// The recording forward keeps one tape per pass, back to back; u is the same in every pass and enters through the
// first one; the operator values and the gradients of the passes add up, always in pass order (bitwise reproducible).
struct PassTapes {
  Split sp;
  std::vector<size_t> off;   // byte offset of each pass's tape
  size_t total;
  int dirs(int pass) const { return pass == sp.n_passes - 1 ? sp.lastR : sp.first; }
};
PassTapes pass_tapes(const ctm_mlp *m, int K, long N, int R) {
  PassTapes t;
  t.sp = split_dirs(K, R);
  size_t off = 0;
  for (int p = 0; p < t.sp.n_passes; ++p) {
    t.off.push_back(off);
    off += tape_layout(m, K, N, t.dirs(p)).total;
  }
  t.total = off;
  return t;
}

template <typename T>
int fwd_tape_passes(const ctm_mlp *m, int K, const T *x, long N, const T *V, int R, long sn, double scale, T *u, T *op, void *tape,
                    hipStream_t st, bool accumulate_first) {
  const PassTapes pt = pass_tapes(m, K, N, R);
  for (int p = 0; p < pt.sp.n_passes; ++p) {
    const bool first = !accumulate_first && p == 0;
    const int rc = run_fwd_tape<T>(m, K, x, N, V, pt.dirs(p), sn, scale, first ? u : nullptr, op, (char *)tape + pt.off[p], st, !first,
                                   p * pt.sp.first);
    if (rc != CTM_OK) return rc;
  }
  return CTM_OK;
}

template <typename T>
int bwd_passes(const ctm_mlp *m, int K, long N, int R, double scale, const void *tape, const T *gu, const T *gop, void *const *gW,
               void *const *gb, void *ws, hipStream_t st, bool accumulate_first) {
  const PassTapes pt = pass_tapes(m, K, N, R);
  for (int p = 0; p < pt.sp.n_passes; ++p) {
    const bool first = !accumulate_first && p == 0;
    const int rc = run_bwd<T>(m, K, N, pt.dirs(p), scale, (const char *)tape + pt.off[p], first ? gu : nullptr, gop, gW, gb, ws, st,
                              first ? 0 : 1);
    if (rc != CTM_OK) return rc;
  }
  return CTM_OK;
}

}  // namespace

extern "C" {

const char *ctm_last_error(void) { return g_err.c_str(); }

int ctm_profile_begin(void) {
  for (hipEvent_t e : g_prof.ev) (void)hipEventDestroy(e);
  g_prof.ev.clear();
  g_prof.cls.clear();
  g_prof.on = true;
  return CTM_OK;
}

int ctm_profile_end(double ms[3], long launches[3]) {
  g_prof.on = false;
  int rc = CTM_OK;
  if (ms) ms[0] = ms[1] = ms[2] = 0.0;
  if (launches) launches[0] = launches[1] = launches[2] = 0;
  if (!g_prof.ev.empty()) {
    hipError_t e = hipEventSynchronize(g_prof.ev.back());
    if (e != hipSuccess) rc = fail_hip(e, "ctm_profile_end: hipEventSynchronize");
    for (size_t i = 0; rc == CTM_OK && i < g_prof.cls.size(); ++i) {
      const int c = g_prof.cls[i];
      if (c < 0) continue;
      float dt = 0.f;
      e = hipEventElapsedTime(&dt, g_prof.ev[i], g_prof.ev[i + 1]);
      if (e != hipSuccess) { rc = fail_hip(e, "ctm_profile_end: hipEventElapsedTime"); break; }
      if (ms) ms[c] += dt;
      if (launches) launches[c] += 1;
    }
  }
  for (hipEvent_t e : g_prof.ev) (void)hipEventDestroy(e);
  g_prof.ev.clear();
  g_prof.cls.clear();
  return rc;
}

long ctm_rows_per_point(int K, int R) {
  if ((K != 2 && K != 4) || R < 1) return -1;
  return rows_per_point(K, R);
}

int ctm_tile_plan(ctm_dtype dtype, int K, int R, int *points_per_tile, int *row_blocks, int *dirs_per_pass,
                  int *n_passes) {
  if (!known_dtype(dtype)) return fail(CTM_ERR_DTYPE, "ctm_tile_plan: unknown dtype %d", (int)dtype);
  if (K != 2 && K != 4) return fail(CTM_ERR_UNSUPPORTED, "ctm_tile_plan: order K = %d, only 2 and 4 are built", K);
  if (R < 1) return fail(CTM_ERR_SHAPE, "ctm_tile_plan: %d directions, need at least 1", R);
  const Split sp = split_dirs(K, R);
  const PassPlan pl = plan_pass(K, sp.first);
  if (points_per_tile) *points_per_tile = pl.P;
  if (row_blocks) *row_blocks = pl.MB;
  if (dirs_per_pass) *dirs_per_pass = sp.first;
  if (n_passes) *n_passes = sp.n_passes;
  return CTM_OK;
}

int ctm_create_mlp(int n_layers, const int *dims, const void *const *W, const void *const *b, ctm_dtype dtype,
                   ctm_act act, void *stream, ctm_mlp **out) {
  if (!out) return fail(CTM_ERR_NULL, "ctm_create_mlp: out is NULL");
  *out = nullptr;
  if (!dims || !W) return fail(CTM_ERR_NULL, "ctm_create_mlp: dims or W is NULL");
  if (!known_dtype(dtype)) return fail(CTM_ERR_DTYPE, "ctm_create_mlp: unknown dtype %d", (int)dtype);
  if (act != CTM_ACT_TANH && act != CTM_ACT_IDENTITY && act != CTM_ACT_SIN)
    return fail(CTM_ERR_DTYPE, "ctm_create_mlp: unknown activation %d", (int)act);
  if (n_layers < 2 || n_layers > 64)
    return fail(CTM_ERR_SHAPE, "ctm_create_mlp: n_layers = %d, need 2..64 (at least one hidden layer)", n_layers);
  for (int l = 0; l <= n_layers; ++l)
    if (dims[l] < 1 || dims[l] > (1 << 20)) return fail(CTM_ERR_SHAPE, "ctm_create_mlp: dims[%d] = %d out of range", l, dims[l]);
  if (dims[n_layers] > kMaxOutputs)
    return fail(CTM_ERR_UNSUPPORTED, "ctm_create_mlp: %d outputs, at most %d are built", dims[n_layers], kMaxOutputs);
  const size_t es = elem_size(dtype);
  for (int l = 0; l < n_layers; ++l) {
    if (!W[l]) return fail(CTM_ERR_NULL, "ctm_create_mlp: W[%d] is NULL", l);
    if (misaligned(W[l], es) || (b && misaligned(b[l], es)))
      return fail(CTM_ERR_ALIGN, "ctm_create_mlp: W[%d] / b[%d] not aligned to the element size", l, l);
  }

  ctm_mlp *m = new (std::nothrow) ctm_mlp;
  if (!m) return fail(CTM_ERR_ALLOC, "ctm_create_mlp: out of host memory");
  m->L = n_layers;
  m->dims.assign(dims, dims + n_layers + 1);
  m->dtype = dtype;
  m->act = act;
  const int bn = tile_cols_of(dtype);
  size_t total = 0;
  std::vector<size_t> woff(n_layers), boff(n_layers), hoff(n_layers, 0), loff(n_layers, 0), toff(n_layers, 0);
  for (int l = 0; l < n_layers; ++l) {
    m->ld.push_back(pad_ld(dims[l]));
    const bool lastl = (l == n_layers - 1);
    const int ct = lastl ? 0 : (dims[l + 1] + bn - 1) / bn;
    if (!lastl) m->col_tiles.push_back(ct);
    const size_t rows_pad = lastl ? (size_t)dims[n_layers] : (size_t)ct * bn;
    woff[l] = total;
    total += round256(rows_pad * m->ld[l] * es);
    boff[l] = total;
    total += round256(rows_pad * es);
    if (is_bf16(dtype) && !lastl) {   // the 256-column plain-bf16 kernel reads whole 256-row column tiles
      const size_t rows_bf = (rows_pad + kWideCols - 1) / kWideCols * kWideCols;
      hoff[l] = total;
      total += round256(rows_bf * m->ld[l] * 2);
      loff[l] = total;
      total += round256(rows_bf * m->ld[l] * 2);
    }
    if (l >= 1 && !lastl) {  // transposed copy: rows = padded dims[l], k extent = ld of dims[l+1]
      toff[l] = total;
      total += round256((size_t)((dims[l] + bn - 1) / bn) * bn * pad_ld(dims[l + 1]) * es);
    }
  }
  const size_t w1t_off = total;  // W_1 transposed, zero-padded to [ld(dims[0])][ld(dims[1])]
  total += round256((size_t)m->ld[0] * m->ld[1] * es);
  hipError_t e = hipGetDevice(&m->device);
  if (e != hipSuccess) { delete m; return fail_hip(e, "ctm_create_mlp: hipGetDevice"); }
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, m->device) == hipSuccess && cus > 0) { m->slots = 2 * cus; m->cus = cus; }
  m->min_col_tiles = m->col_tiles[0];
  for (int ct : m->col_tiles) m->min_col_tiles = ct < m->min_col_tiles ? ct : m->min_col_tiles;
  e = hipMalloc(&m->arena, total);
  if (e != hipSuccess) {
    delete m;
    (void)hipGetLastError();
    return fail(CTM_ERR_ALLOC, "ctm_create_mlp: hipMalloc of %zu bytes failed: %s", total, hipGetErrorString(e));
  }
  for (int l = 0; l < n_layers; ++l) {
    m->Wp.push_back((char *)m->arena + woff[l]);
    m->bp.push_back((char *)m->arena + boff[l]);
    m->Whi.push_back((char *)m->arena + hoff[l]);
    m->Wlo.push_back((char *)m->arena + loff[l]);
    m->WT.push_back((char *)m->arena + toff[l]);
  }
  m->W1T = (char *)m->arena + w1t_off;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  e = pack_everything(m, W, b, st);
  if (e != hipSuccess) {
    (void)hipFree(m->arena);
    delete m;
    return fail_hip(e, "ctm_create_mlp: weight packing");
  }
  *out = m;
  return CTM_OK;
}

int ctm_destroy_mlp(ctm_mlp *m) {
  if (!m) return CTM_OK;
  int rc = CTM_OK;
  hipError_t e = hipDeviceSynchronize();
  if (e != hipSuccess) rc = fail_hip(e, "ctm_destroy_mlp: hipDeviceSynchronize");
  e = hipFree(m->arena);
  if (e != hipSuccess && rc == CTM_OK) rc = fail_hip(e, "ctm_destroy_mlp: hipFree");
  delete m;
  return rc;
}

size_t ctm_workspace_bytes(const ctm_mlp *m, int K, long N, int R) {
  if (!m) { fail(CTM_ERR_NULL, "ctm_workspace_bytes: mlp handle is NULL"); return 0; }
  if ((K != 2 && K != 4) || N < 1 || R < 1) {
    fail(CTM_ERR_SHAPE, "ctm_workspace_bytes: need K in {2,4}, N >= 1, R >= 1 (got %d, %ld, %d)", K, N, R);
    return 0;
  }
  return workspace_layout(m, K, N, split_dirs(K, R).first).total;
}

size_t ctm_workspace_bytes_standard(const ctm_mlp *m, int K, long N, int R) {
  if (!m) { fail(CTM_ERR_NULL, "ctm_workspace_bytes_standard: mlp handle is NULL"); return 0; }
  if ((K != 2 && K != 4) || N < 1 || R < 1) {
    fail(CTM_ERR_SHAPE, "ctm_workspace_bytes_standard: need K in {2,4}, N >= 1, R >= 1 (got %d, %ld, %d)", K, N, R);
    return 0;
  }
  return workspace_layout(m, K, N, split_dirs(K, R, true).first, true).total;
}

int ctm_taylor_standard(const ctm_mlp *m, int K, const void *x, long N, const void *V, int R, long v_point_stride,
                        double scale, void *u, void *op, void *ws, size_t ws_bytes, void *stream) {
  const char *who = "ctm_taylor_standard";
  if (K != 2 && K != 4) return fail(CTM_ERR_UNSUPPORTED, "%s: order K = %d, only 2 and 4 are built", who, K);
  if (m && !V && R != m->dims[0])
    return fail(CTM_ERR_SHAPE, "%s: V = NULL selects the standard basis, so R must be D = %d (got %d)", who, m->dims[0], R);
  if (m && R >= 1 && v_point_stride != 0 && v_point_stride != (long)R * m->dims[0])
    return fail(CTM_ERR_SHAPE, "%s: v_point_stride = %ld, must be 0 (shared) or R*D = %ld", who, v_point_stride,
                (long)R * m->dims[0]);
  const long D = m ? m->dims[0] : 0;
  return run_operator(m, K, x, N, V, R, v_point_stride, D, 1, scale, u, op, ws, ws_bytes, stream, who, true);
}

int ctm_laplacian(const ctm_mlp *m, const void *x, long N, const void *V, int R, long v_point_stride, double scale,
                  void *u, void *op, void *ws, size_t ws_bytes, void *stream) {
  if (m && !V && R != m->dims[0])
    return fail(CTM_ERR_SHAPE, "ctm_laplacian: V = NULL selects the standard basis, so R must be D = %d (got %d)", m->dims[0], R);
  if (m && R >= 1 && v_point_stride != 0 && v_point_stride != (long)R * m->dims[0])
    return fail(CTM_ERR_SHAPE, "ctm_laplacian: v_point_stride = %ld, must be 0 (shared) or R*D = %ld", v_point_stride,
                (long)R * m->dims[0]);
  const long D = m ? m->dims[0] : 0;
  return run_operator(m, 2, x, N, V, R, v_point_stride, D, 1, scale, u, op, ws, ws_bytes, stream, "ctm_laplacian");
}

int ctm_laplacian_static(const ctm_mlp *m, const void *x, long N, const void *V, int R, long v_point_stride, double scale,
                         void *u, void *op, void *stream) {
  const char *who = "ctm_laplacian_static";
  if (!m) return fail(CTM_ERR_NULL, "%s: mlp handle is NULL", who);
  if (N < 1) return fail(CTM_ERR_SHAPE, "%s: N = %ld, need N >= 1", who, N);
  if (R < 1) return fail(CTM_ERR_SHAPE, "%s: %d directions, need at least 1", who, R);
  if (!V && R != m->dims[0])
    return fail(CTM_ERR_SHAPE, "%s: V = NULL selects the standard basis, so R must be D = %d (got %d)", who, m->dims[0], R);
  if (v_point_stride != 0 && v_point_stride != (long)R * m->dims[0])
    return fail(CTM_ERR_SHAPE, "%s: v_point_stride = %ld, must be 0 (shared) or R*D = %ld", who, v_point_stride,
                (long)R * m->dims[0]);
  if (N > (1L << 40) / rows_per_point(2, R)) return fail(CTM_ERR_SHAPE, "%s: N * rows per point overflows", who);
  const size_t need = workspace_layout(m, 2, N, split_dirs(2, R).first).total;
  if (need > (size_t)CTM_STATIC_SCRATCH_BYTES)
    return fail(CTM_ERR_WORKSPACE,
                "%s: N = %ld points with %d directions need %zu bytes of scratch, the built-in array holds %zu; "
                "use ctm_laplacian with a workspace of your own",
                who, N, R, need, (size_t)CTM_STATIC_SCRATCH_BYTES);
  if (int rc = check_device(m, who)) return rc;
  void *ws = nullptr;
  if (int rc = static_scratch(m->device, who, &ws)) return rc;
  return run_operator(m, 2, x, N, V, R, v_point_stride, m->dims[0], 1, scale, u, op, ws, (size_t)CTM_STATIC_SCRATCH_BYTES,
                      stream, who);
}

int ctm_weighted_laplacian(const ctm_mlp *m, const void *x, long N, const void *sigma, int K, void *u, void *op,
                           void *ws, size_t ws_bytes, void *stream) {
  if (m && !sigma) return fail(CTM_ERR_NULL, "ctm_weighted_laplacian: sigma is NULL");
  // direction k is column k of sigma[D][K]: element (k, d) sits at sigma[d*K + k]
  return run_operator(m, 2, x, N, sigma, K, 0, 1, K, 1.0, u, op, ws, ws_bytes, stream, "ctm_weighted_laplacian");
}

int ctm_biharmonic_rand(const ctm_mlp *m, const void *x, long N, const void *V, int S, long v_point_stride, void *u,
                        void *op, void *ws, size_t ws_bytes, void *stream) {
  if (m && !V) return fail(CTM_ERR_NULL, "ctm_biharmonic_rand: V is NULL");
  if (m && S >= 1 && v_point_stride != 0 && v_point_stride != (long)S * m->dims[0])
    return fail(CTM_ERR_SHAPE, "ctm_biharmonic_rand: v_point_stride = %ld, must be 0 (shared) or S*D = %ld",
                v_point_stride, (long)S * m->dims[0]);
  const long D = m ? m->dims[0] : 0;
  const double scale = S >= 1 ? 1.0 / (3.0 * S) : 0.0;
  return run_operator(m, 4, x, N, V, S, v_point_stride, D, 1, scale, u, op, ws, ws_bytes, stream, "ctm_biharmonic_rand");
}

size_t ctm_weighted_laplacian_rand_workspace_bytes(const ctm_mlp *m, long N, int K, int S, long sigma_point_stride,
                                                   long v_point_stride) {
  if (!m) { fail(CTM_ERR_NULL, "ctm_weighted_laplacian_rand_workspace_bytes: mlp handle is NULL"); return 0; }
  if (N < 1 || K < 1 || S < 0) {
    fail(CTM_ERR_SHAPE, "ctm_weighted_laplacian_rand_workspace_bytes: need N >= 1, K >= 1, S >= 0");
    return 0;
  }
  const int R = S > 0 ? S : K;
  const size_t base = workspace_layout(m, 2, N, split_dirs(2, R).first).total;
  if (S == 0) return base;  // exact: the directions are columns of sigma, read in place
  const bool per_point = sigma_point_stride != 0 || v_point_stride != 0;
  return base + round256((size_t)(per_point ? N : 1) * S * m->dims[0] * elem_size(m->dtype));
}

int ctm_weighted_laplacian_rand(const ctm_mlp *m, const void *x, long N, const void *sigma, int K, long sigma_point_stride,
                                const void *V, int S, long v_point_stride, void *u, void *op, void *ws, size_t ws_bytes,
                                void *stream) {
  const char *who = "ctm_weighted_laplacian_rand";
  if (!m) return fail(CTM_ERR_NULL, "%s: mlp handle is NULL", who);
  if (!sigma) return fail(CTM_ERR_NULL, "%s: sigma is NULL", who);
  if (K < 1) return fail(CTM_ERR_SHAPE, "%s: sigma has %d columns, need at least 1", who, K);
  const long D = m->dims[0];
  if (sigma_point_stride != 0 && sigma_point_stride != D * K)
    return fail(CTM_ERR_SHAPE, "%s: sigma_point_stride = %ld, must be 0 (shared) or D*K = %ld", who, sigma_point_stride, D * K);
  if (!V) {
    if (S != 0) return fail(CTM_ERR_SHAPE, "%s: V = NULL selects the exact operator, so S must be 0 (got %d)", who, S);
    // directions are the K columns of sigma_n: element (n, k, d) at sigma[n*stride + d*K + k]
    return run_operator(m, 2, x, N, sigma, K, sigma_point_stride, 1, K, 1.0, u, op, ws, ws_bytes, stream, who);
  }
  if (S < 1) return fail(CTM_ERR_SHAPE, "%s: %d samples, need at least 1", who, S);
  if (v_point_stride != 0 && v_point_stride != (long)S * K)
    return fail(CTM_ERR_SHAPE, "%s: v_point_stride = %ld, must be 0 (shared) or S*K = %ld", who, v_point_stride, (long)S * K);
  if (N < 1) return fail(CTM_ERR_SHAPE, "%s: N = %ld, need N >= 1", who, N);
  if (!ws) return fail(CTM_ERR_NULL, "%s: workspace is NULL", who);
  const size_t need = ctm_weighted_laplacian_rand_workspace_bytes(m, N, K, S, sigma_point_stride, v_point_stride);
  if (ws_bytes < need) return fail(CTM_ERR_WORKSPACE, "%s: workspace has %zu bytes, need %zu", who, ws_bytes, need);
  const size_t es = elem_size(m->dtype);
  if (misaligned(ws, 256)) return fail(CTM_ERR_ALIGN, "%s: workspace must be 256-byte aligned", who);
  if (misaligned(sigma, es) || misaligned(V, es))
    return fail(CTM_ERR_ALIGN, "%s: sigma and V must be aligned to the element size", who);
  // everything run_operator would refuse is refused here, before the direction kernel is queued
  if (!x) return fail(CTM_ERR_NULL, "%s: x is NULL", who);
  if (N > (1L << 40) / rows_per_point(2, S)) return fail(CTM_ERR_SHAPE, "%s: N * rows per point overflows", who);
  if (misaligned(x, es) || misaligned(u, es) || misaligned(op, es))
    return fail(CTM_ERR_ALIGN, "%s: x, u and op must be aligned to the element size", who);
  const bool per_point = sigma_point_stride != 0 || v_point_stride != 0;
  const long Nd = per_point ? N : 1;
  const size_t dbytes = round256((size_t)Nd * S * D * es);
  if (int rc = check_device(m, who)) return rc;
  void *dirs = (char *)ws + (need - dbytes);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  hipError_t e = (m->dtype == CTM_F64)
                     ? launch_sigma_dirs<double>((const double *)sigma, sigma_point_stride, (const double *)V, v_point_stride,
                                                 (double *)dirs, Nd, S, (int)D, K, st)
                     : launch_sigma_dirs<float>((const float *)sigma, sigma_point_stride, (const float *)V, v_point_stride,
                                                (float *)dirs, Nd, S, (int)D, K, st);
  if (e != hipSuccess) return fail_hip(e, "direction kernel launch");
  return run_operator(m, 2, x, N, dirs, S, per_point ? (long)S * D : 0, D, 1, 1.0 / S, u, op, ws, need - dbytes, stream, who);
}

int ctm_update_mlp(ctm_mlp *m, const void *const *W, const void *const *b, void *stream) {
  if (!m || !W) return fail(CTM_ERR_NULL, "ctm_update_mlp: mlp handle or W is NULL");
  const size_t es = elem_size(m->dtype);
  for (int l = 0; l < m->L; ++l) {
    if (!W[l]) return fail(CTM_ERR_NULL, "ctm_update_mlp: W[%d] is NULL", l);
    if (misaligned(W[l], es) || (b && misaligned(b[l], es)))
      return fail(CTM_ERR_ALIGN, "ctm_update_mlp: W[%d] / b[%d] not aligned to the element size", l, l);
  }
  if (int rc = check_device(m, "ctm_update_mlp")) return rc;
  {
    std::lock_guard<std::mutex> g(m->mu);
    ++m->version;
  }
  hipError_t e = pack_everything(m, W, b, reinterpret_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail_hip(e, "ctm_update_mlp: weight packing");
  return CTM_OK;
}

size_t ctm_tape_bytes(const ctm_mlp *m, long N, int R) {
  if (check_tape_call(m, 2, N, R, "ctm_tape_bytes") != CTM_OK) return 0;
  return pass_tapes(m, 2, N, R).total;
}

size_t ctm_backward_workspace_bytes(const ctm_mlp *m, long N, int R) {
  if (check_tape_call(m, 2, N, R, "ctm_backward_workspace_bytes") != CTM_OK) return 0;
  return bwd_layout(m, 2, N, split_dirs(2, R).first).total;
}

size_t ctm_biharmonic_tape_bytes(const ctm_mlp *m, long N, int S) {
  if (check_tape_call(m, 4, N, S, "ctm_biharmonic_tape_bytes") != CTM_OK) return 0;
  return pass_tapes(m, 4, N, S).total;
}

size_t ctm_biharmonic_backward_workspace_bytes(const ctm_mlp *m, long N, int S) {
  if (check_tape_call(m, 4, N, S, "ctm_biharmonic_backward_workspace_bytes") != CTM_OK) return 0;
  return bwd_layout(m, 4, N, split_dirs(4, S).first).total;
}

}  // extern "C"

namespace {

int recording_forward(const char *who, const ctm_mlp *m, int K, const void *x, long N, const void *V, int R, long v_point_stride,
                      double scale, void *u, void *op, void *tape, size_t tape_bytes, void *stream) {
  int rc = check_tape_call(m, K, N, R, who);
  if (rc != CTM_OK) return rc;
  if (!x || !tape) return fail(CTM_ERR_NULL, "%s: x or tape is NULL", who);
  if (K == 4 && !V) return fail(CTM_ERR_NULL, "%s: V is NULL", who);
  if (!V && R != m->dims[0]) return fail(CTM_ERR_SHAPE, "%s: V = NULL selects the standard basis, so R must be D = %d (got %d)", who, m->dims[0], R);
  if (v_point_stride != 0 && v_point_stride != (long)R * m->dims[0])
    return fail(CTM_ERR_SHAPE, "%s: v_point_stride = %ld, must be 0 (shared) or R*D = %ld", who, v_point_stride, (long)R * m->dims[0]);
  const size_t need = pass_tapes(m, K, N, R).total;
  if (tape_bytes < need) return fail(CTM_ERR_WORKSPACE, "%s: tape has %zu bytes, need %zu", who, tape_bytes, need);
  const size_t es = elem_size(m->dtype);
  if (misaligned(tape, 256)) return fail(CTM_ERR_ALIGN, "%s: tape must be 256-byte aligned", who);
  if (misaligned(x, es) || misaligned(V, es) || misaligned(u, es) || misaligned(op, es))
    return fail(CTM_ERR_ALIGN, "%s: x, directions, u and op must be aligned to the element size", who);
  if (int rc2 = check_device(m, who)) return rc2;
  m->note_tape(tape);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (m->dtype == CTM_F64)
    return fwd_tape_passes<double>(m, K, (const double *)x, N, (const double *)V, R, v_point_stride, scale, (double *)u, (double *)op, tape, st, false);
  return fwd_tape_passes<float>(m, K, (const float *)x, N, (const float *)V, R, v_point_stride, scale, (float *)u, (float *)op, tape, st, false);
}

int reverse_pass(const char *who, const ctm_mlp *m, int K, long N, int R, double scale, const void *tape, size_t tape_bytes,
                 const void *gu, const void *gop, void *const *gW, void *const *gb, void *ws, size_t ws_bytes, void *stream) {
  int rc = check_tape_call(m, K, N, R, who);
  if (rc != CTM_OK) return rc;
  if (!tape || !ws) return fail(CTM_ERR_NULL, "%s: tape or workspace is NULL", who);
  if (tape_bytes < pass_tapes(m, K, N, R).total) return fail(CTM_ERR_WORKSPACE, "%s: tape is smaller than the tape size query says", who);
  const size_t need = bwd_layout(m, K, N, split_dirs(K, R).first).total;
  if (ws_bytes < need) return fail(CTM_ERR_WORKSPACE, "%s: workspace has %zu bytes, need %zu", who, ws_bytes, need);
  const size_t es = elem_size(m->dtype);
  if (misaligned(tape, 256) || misaligned(ws, 256)) return fail(CTM_ERR_ALIGN, "%s: tape and workspace must be 256-byte aligned", who);
  if (misaligned(gu, es) || misaligned(gop, es)) return fail(CTM_ERR_ALIGN, "%s: gu and gop must be aligned to the element size", who);
  for (int l = 0; l < m->L; ++l)
    if ((gW && misaligned(gW[l], es)) || (gb && misaligned(gb[l], es)))
      return fail(CTM_ERR_ALIGN, "%s: gW[%d] / gb[%d] not aligned to the element size", who, l, l);
  if (int rc2 = check_device(m, who)) return rc2;
  if (!m->tape_matches(tape))
    return fail(CTM_ERR_UNSUPPORTED, "%s: the handle's weights were replaced (ctm_update_mlp) after the forward call that recorded this tape", who);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  if (m->dtype == CTM_F64)
    return bwd_passes<double>(m, K, N, R, scale, tape, (const double *)gu, (const double *)gop, gW, gb, ws, st, false);
  return bwd_passes<float>(m, K, N, R, scale, tape, (const float *)gu, (const float *)gop, gW, gb, ws, st, false);
}

}  // namespace

extern "C" {

int ctm_laplacian_fwd(const ctm_mlp *m, const void *x, long N, const void *V, int R, long v_point_stride, double scale, void *u,
                      void *op, void *tape, size_t tape_bytes, void *stream) {
  return recording_forward("ctm_laplacian_fwd", m, 2, x, N, V, R, v_point_stride, scale, u, op, tape, tape_bytes, stream);
}

int ctm_laplacian_bwd(const ctm_mlp *m, long N, int R, double scale, const void *tape, size_t tape_bytes, const void *gu,
                      const void *gop, void *const *gW, void *const *gb, void *ws, size_t ws_bytes, void *stream) {
  return reverse_pass("ctm_laplacian_bwd", m, 2, N, R, scale, tape, tape_bytes, gu, gop, gW, gb, ws, ws_bytes, stream);
}

int ctm_biharmonic_rand_fwd(const ctm_mlp *m, const void *x, long N, const void *V, int S, long v_point_stride, void *u, void *op,
                            void *tape, size_t tape_bytes, void *stream) {
  const double scale = S >= 1 ? 1.0 / (3.0 * S) : 0.0;
  return recording_forward("ctm_biharmonic_rand_fwd", m, 4, x, N, V, S, v_point_stride, scale, u, op, tape, tape_bytes, stream);
}

int ctm_biharmonic_rand_bwd(const ctm_mlp *m, long N, int S, const void *tape, size_t tape_bytes, const void *gu, const void *gop,
                            void *const *gW, void *const *gb, void *ws, size_t ws_bytes, void *stream) {
  const double scale = S >= 1 ? 1.0 / (3.0 * S) : 0.0;
  return reverse_pass("ctm_biharmonic_rand_bwd", m, 4, N, S, scale, tape, tape_bytes, gu, gop, gW, gb, ws, ws_bytes, stream);
}

int ctm_interpolation_gamma(int I, const int *i, const int *j, long long *num, long long *den) {
  if (!i || !j || !num || !den) return fail(CTM_ERR_NULL, "ctm_interpolation_gamma: NULL argument");
  if (I < 1 || I > 4) return fail(CTM_ERR_SHAPE, "ctm_interpolation_gamma: I = %d, need 1..4", I);
  int si = 0, sj = 0;
  for (int t = 0; t < I; ++t) {
    if (i[t] < 0 || j[t] < 0 || i[t] > 8 || j[t] > 8) return fail(CTM_ERR_SHAPE, "ctm_interpolation_gamma: entries must lie in 0..8");
    si += i[t];
    sj += j[t];
  }
  if (si != sj || si < 1 || si > 8) return fail(CTM_ERR_SHAPE, "ctm_interpolation_gamma: |i| = %d and |j| = %d must agree and lie in 1..8", si, sj);
  g_frac_overflow = false;
  const Frac g = interp_gamma(I, i, j);
  if (g_frac_overflow) return fail(CTM_ERR_UNSUPPORTED, "ctm_interpolation_gamma: an intermediate fraction does not fit 64 bits");
  *num = g.n;
  *den = g.d;
  return CTM_OK;
}

size_t ctm_biharmonic_exact_workspace_bytes(const ctm_mlp *m, long N) {
  if (!m) { fail(CTM_ERR_NULL, "ctm_biharmonic_exact_workspace_bytes: mlp handle is NULL"); return 0; }
  if (N < 1) { fail(CTM_ERR_SHAPE, "ctm_biharmonic_exact_workspace_bytes: N = %ld, need N >= 1", N); return 0; }
  const long D = m->dims[0];
  const long rmax = D > 1 ? D * (D - 1) : D;
  if (rmax > 0x7fffffffL) { fail(CTM_ERR_SHAPE, "ctm_biharmonic_exact_workspace_bytes: D too large"); return 0; }
  return workspace_layout(m, 4, N, split_dirs(4, (int)rmax).first).total + round256((size_t)rmax * D * elem_size(m->dtype));
}

}  // extern "C"

namespace {

// The three direction families of the interpolation formula (Sec. 3.3, Eq. 12; App. E.1, last display) and their weights.
struct BiharmFamilies {
  double weight[3];
  long count[3];
  long rmax;
};
BiharmFamilies biharm_families(int D) {
  const int i22[2] = {2, 2}, j40[2] = {4, 0}, j31[2] = {3, 1}, j22[2] = {2, 2};
  const Frac g40 = interp_gamma(2, i22, j40), g31 = interp_gamma(2, i22, j31), g22 = interp_gamma(2, i22, j22);
  const double G40 = (double)g40.n / g40.d, G31 = (double)g31.n / g31.d, G22 = (double)g22.n / g22.d;
  BiharmFamilies f;
  f.weight[0] = (2.0 * D * G40 + 2.0 * G31 + G22) / 24.0;
  f.weight[1] = 2.0 * G31 / 24.0;
  f.weight[2] = 2.0 * G22 / 24.0;
  f.count[0] = D;
  f.count[1] = (long)D * (D - 1);
  f.count[2] = (long)D * (D - 1) / 2;
  f.rmax = D > 1 ? (long)D * (D - 1) : D;
  return f;
}

// Tape of the differentiable exact biharmonic: one order-4 tape per family, then the direction scratch.
struct ExactTape {
  size_t off[3], dirs, total;
};
int exact_tape_layout(const ctm_mlp *m, long N, const char *who, ExactTape *t) {
  if (!m) return fail(CTM_ERR_NULL, "%s: mlp handle is NULL", who);
  const BiharmFamilies f = biharm_families(m->dims[0]);
  size_t off = 0;
  for (int fam = 0; fam < 3; ++fam) {
    t->off[fam] = off;
    if (f.count[fam] == 0) continue;
    if (f.count[fam] > 0x7fffffffL) return fail(CTM_ERR_SHAPE, "%s: D too large", who);
    const int rc = check_tape_call(m, 4, N, (int)f.count[fam], who);
    if (rc != CTM_OK) return rc;
    off += pass_tapes(m, 4, N, (int)f.count[fam]).total;
  }
  t->dirs = off;
  t->total = off + round256((size_t)f.rmax * m->dims[0] * elem_size(m->dtype));
  return CTM_OK;
}

// Reverse-pass workspace of the exact biharmonic: the largest pass of any family.
size_t exact_bwd_need(const ctm_mlp *m, long N) {
  const BiharmFamilies f = biharm_families(m->dims[0]);
  size_t need = 0;
  for (int fam = 0; fam < 3; ++fam) {
    if (f.count[fam] == 0) continue;
    const size_t b = bwd_layout(m, 4, N, split_dirs(4, (int)f.count[fam]).first).total;
    need = b > need ? b : need;
  }
  return need;
}

}  // namespace

extern "C" {

size_t ctm_biharmonic_exact_tape_bytes(const ctm_mlp *m, long N) {
  ExactTape t;
  return exact_tape_layout(m, N, "ctm_biharmonic_exact_tape_bytes", &t) == CTM_OK ? t.total : 0;
}

size_t ctm_biharmonic_exact_backward_workspace_bytes(const ctm_mlp *m, long N) {
  ExactTape t;
  if (exact_tape_layout(m, N, "ctm_biharmonic_exact_backward_workspace_bytes", &t) != CTM_OK) return 0;
  return exact_bwd_need(m, N);
}

int ctm_biharmonic_exact_fwd(const ctm_mlp *m, const void *x, long N, void *u, void *op, void *tape, size_t tape_bytes,
                             void *stream) {
  const char *who = "ctm_biharmonic_exact_fwd";
  ExactTape t;
  int rc = exact_tape_layout(m, N, who, &t);
  if (rc != CTM_OK) return rc;
  if (!x || !tape) return fail(CTM_ERR_NULL, "%s: x or tape is NULL", who);
  if (tape_bytes < t.total) return fail(CTM_ERR_WORKSPACE, "%s: tape has %zu bytes, need %zu", who, tape_bytes, t.total);
  const size_t es = elem_size(m->dtype);
  if (misaligned(tape, 256)) return fail(CTM_ERR_ALIGN, "%s: tape must be 256-byte aligned", who);
  if (misaligned(x, es) || misaligned(u, es) || misaligned(op, es))
    return fail(CTM_ERR_ALIGN, "%s: x, u and op must be aligned to the element size", who);
  if ((rc = check_device(m, who)) != CTM_OK) return rc;
  m->note_tape(tape);
  const int D = m->dims[0];
  const BiharmFamilies f = biharm_families(D);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  char *tp = (char *)tape;
  bool first = true;
  for (int fam = 0; fam < 3; ++fam) {
    if (f.count[fam] == 0) continue;
    if (m->dtype == CTM_F64) {
      hipError_t e = launch_biharm_dirs<double>((double *)(tp + t.dirs), D, fam, st);
      if (e != hipSuccess) return fail_hip(e, "direction kernel launch");
      rc = fwd_tape_passes<double>(m, 4, (const double *)x, N, (const double *)(tp + t.dirs), (int)f.count[fam], 0, f.weight[fam],
                                   (double *)u, (double *)op, tp + t.off[fam], st, !first);
    } else {
      hipError_t e = launch_biharm_dirs<float>((float *)(tp + t.dirs), D, fam, st);
      if (e != hipSuccess) return fail_hip(e, "direction kernel launch");
      rc = fwd_tape_passes<float>(m, 4, (const float *)x, N, (const float *)(tp + t.dirs), (int)f.count[fam], 0, f.weight[fam],
                                  (float *)u, (float *)op, tp + t.off[fam], st, !first);
    }
    if (rc != CTM_OK) return rc;
    first = false;
  }
  return CTM_OK;
}

int ctm_biharmonic_exact_bwd(const ctm_mlp *m, long N, const void *tape, size_t tape_bytes, const void *gu, const void *gop,
                             void *const *gW, void *const *gb, void *ws, size_t ws_bytes, void *stream) {
  const char *who = "ctm_biharmonic_exact_bwd";
  ExactTape t;
  int rc = exact_tape_layout(m, N, who, &t);
  if (rc != CTM_OK) return rc;
  if (!tape || !ws) return fail(CTM_ERR_NULL, "%s: tape or workspace is NULL", who);
  if (tape_bytes < t.total) return fail(CTM_ERR_WORKSPACE, "%s: tape is smaller than ctm_biharmonic_exact_tape_bytes() says", who);
  const BiharmFamilies f = biharm_families(m->dims[0]);
  const size_t need = exact_bwd_need(m, N);
  if (ws_bytes < need) return fail(CTM_ERR_WORKSPACE, "%s: workspace has %zu bytes, need %zu", who, ws_bytes, need);
  const size_t es = elem_size(m->dtype);
  if (misaligned(tape, 256) || misaligned(ws, 256)) return fail(CTM_ERR_ALIGN, "%s: tape and workspace must be 256-byte aligned", who);
  if (misaligned(gu, es) || misaligned(gop, es)) return fail(CTM_ERR_ALIGN, "%s: gu and gop must be aligned to the element size", who);
  for (int l = 0; l < m->L; ++l)
    if ((gW && misaligned(gW[l], es)) || (gb && misaligned(gb[l], es)))
      return fail(CTM_ERR_ALIGN, "%s: gW[%d] / gb[%d] not aligned to the element size", who, l, l);
  if ((rc = check_device(m, who)) != CTM_OK) return rc;
  if (!m->tape_matches(tape))
    return fail(CTM_ERR_UNSUPPORTED, "%s: the handle's weights were replaced (ctm_update_mlp) after the forward call that recorded this tape", who);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const char *tp = (const char *)tape;
  bool first = true;
  for (int fam = 0; fam < 3; ++fam) {  // the families' contributions add up in this order; u enters through the first only
    if (f.count[fam] == 0) continue;
    if (m->dtype == CTM_F64)
      rc = bwd_passes<double>(m, 4, N, (int)f.count[fam], f.weight[fam], tp + t.off[fam], (const double *)gu, (const double *)gop, gW,
                              gb, ws, st, !first);
    else
      rc = bwd_passes<float>(m, 4, N, (int)f.count[fam], f.weight[fam], tp + t.off[fam], (const float *)gu, (const float *)gop, gW, gb,
                             ws, st, !first);
    if (rc != CTM_OK) return rc;
    first = false;
  }
  return CTM_OK;
}

int ctm_biharmonic_exact(const ctm_mlp *m, const void *x, long N, void *u, void *op, void *ws, size_t ws_bytes,
                         void *stream) {
  const char *who = "ctm_biharmonic_exact";
  if (!m) return fail(CTM_ERR_NULL, "%s: mlp handle is NULL", who);
  if (!x) return fail(CTM_ERR_NULL, "%s: x is NULL", who);
  if (N < 1) return fail(CTM_ERR_SHAPE, "%s: N = %ld, need N >= 1", who, N);
  if (!ws) return fail(CTM_ERR_NULL, "%s: workspace is NULL", who);
  const size_t need = ctm_biharmonic_exact_workspace_bytes(m, N);
  if (need == 0) return CTM_ERR_SHAPE;
  if (ws_bytes < need) return fail(CTM_ERR_WORKSPACE, "%s: workspace has %zu bytes, need %zu", who, ws_bytes, need);
  const size_t es = elem_size(m->dtype);
  if (misaligned(ws, 256)) return fail(CTM_ERR_ALIGN, "%s: workspace must be 256-byte aligned", who);
  if (misaligned(x, es) || misaligned(u, es) || misaligned(op, es))
    return fail(CTM_ERR_ALIGN, "%s: x, u and op must be aligned to the element size", who);
  if (int rc = check_device(m, who)) return rc;
  const int D = m->dims[0];
  // weights of the three direction families (final form of the interpolation formula, App. E.1)
  const BiharmFamilies fams = biharm_families(D);
  const double *weight = fams.weight;
  const long *count = fams.count;
  const long rmax = fams.rmax;
  const size_t vbytes = round256((size_t)rmax * D * es);
  void *vbuf = (char *)ws + (need - vbytes);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  bool first = true;
  for (int fam = 0; fam < 3; ++fam) {
    if (count[fam] == 0) continue;
    int rc;
    if (m->dtype == CTM_F64) {
      hipError_t e = launch_biharm_dirs<double>((double *)vbuf, D, fam, st);
      if (e != hipSuccess) return fail_hip(e, "direction kernel launch");
      rc = run_passes<double>(m, 4, (const double *)x, N, (const double *)vbuf, (int)count[fam], 0, D, 1, weight[fam],
                              first ? (double *)u : nullptr, (double *)op, ws, st, !first);
    } else {
      hipError_t e = launch_biharm_dirs<float>((float *)vbuf, D, fam, st);
      if (e != hipSuccess) return fail_hip(e, "direction kernel launch");
      rc = run_passes<float>(m, 4, (const float *)x, N, (const float *)vbuf, (int)count[fam], 0, D, 1, weight[fam],
                             first ? (float *)u : nullptr, (float *)op, ws, st, !first);
    }
    if (rc != CTM_OK) return rc;
    first = false;
  }
  return CTM_OK;
}

}  // extern "C"
