// The collapsed (or, for comparison, un-collapsed) Taylor-mode rule of the activation for one
// (point, feature) pair: shared by the fp32/fp64 and the bf16-MFMA stacked-GEMM kernels.
//
//   order 2:  t = phi(z_0) ; d1, d2, ... its derivatives (tanh: d1 = 1 - t^2, d2 = -2 t d1, App. H)
//             h_0 = t ;  h_{1,r} = d1 z_{1,r} ;  h_2 = d1 z_2 + d2 * sum_r z_{1,r}^2      (Sec. 3.1, Eq. 6)
//   order 4:  (tanh: d3 = d1 (6 t^2 - 2) ; d4 = 8 t d1 (2 - 3 t^2))
//             h_{1,r} = d1 z1 ; h_{2,r} = d2 z1^2 + d1 z2 ; h_{3,r} = d3 z1^3 + 3 d2 z1 z2 + d1 z3
//             h_4 = d1 z_4 + sum_r [ d4 z1^4 + 6 d3 z1^2 z2 + 4 d2 z1 z3 + 3 d2 z2^2 ]     (App. A multiplicities)
#pragma once

#include "ctm_internal.h"

namespace ctm {

__device__ __forceinline__ float act_tanh(float z) { return tanhf(z); }
__device__ __forceinline__ double act_tanh(double z) { return tanh(z); }
__device__ __forceinline__ void act_sincos(float z, float &s, float &c) { s = sinf(z); c = cosf(z); }
__device__ __forceinline__ void act_sincos(double z, double &s, double &c) { s = sin(z); c = cos(z); }

// Activation value t = phi(z) and first derivative d1; the higher derivatives follow from (t, d1):
//   act 0, tanh:     d1 = 1 - t^2, d2 = -2 t d1, d3 = d1 (6 t^2 - 2), d4 = 8 t d1 (2 - 3 t^2),
//                    d5 = d1 (16 - 120 t^2 + 120 t^4)   (only the reverse of the order-4 rule needs it)
//   act 1, identity: d1 = 1, d2 = d3 = d4 = d5 = 0
//   act 2, sin:      t = sin z, d1 = cos z, d2 = -t, d3 = -d1, d4 = t, d5 = d1
template <typename T> __device__ __forceinline__ void act_eval(int act, T z, T &t, T &d1) {
  if (act == 0) {
    t = act_tanh(z);
    d1 = T(1) - t * t;
  } else if (act == 2) {
    act_sincos(z, t, d1);
  } else {
    t = z;
    d1 = T(1);
  }
}
template <typename T> __device__ __forceinline__ T act_d2(int act, T t, T d1) {
  return act == 0 ? T(-2) * t * d1 : (act == 2 ? -t : T(0));
}
template <typename T> __device__ __forceinline__ T act_d3(int act, T t, T d1) {
  return act == 0 ? d1 * (T(6) * t * t - T(2)) : (act == 2 ? -d1 : T(0));
}
template <typename T> __device__ __forceinline__ T act_d4(int act, T t, T d1) {
  return act == 0 ? T(8) * t * d1 * (T(2) - T(3) * t * t) : (act == 2 ? t : T(0));
}

template <typename T> __device__ __forceinline__ T act_d5(int act, T t, T d1) {
  const T t2 = t * t;
  return act == 0 ? d1 * (T(16) + T(120) * t2 * (t2 - T(1))) : (act == 2 ? d1 : T(0));
}

// Where the rule's output rows go: `put(row, v)` stores the value of coefficient row `row` of the pair's column.
// The column's address is `o` plus `lane_bytes`.  A caller whose wavefront works on one point passes a wavefront-uniform
// `o` (the point's row 0 at the wavefront's first column) and the lane's column in `lane_bytes`: the row address is then
// scalar arithmetic and the store takes it from SGPRs, which keeps 64-bit vector adds out of the rule's loop (vector-ALU
// instructions of the rule take issue cycles away from the MFMAs of the workgroup that shares the CU).
template <typename T> struct PlainRows {  // rows of T, `step` elements apart
  T *o;
  long step;
  mutable unsigned lane_bytes = 0;
  __device__ __forceinline__ void put(long row, T v) const { store(row_base(row), lane_bytes, v); }
  // the pieces of put(), for loops that keep the row address themselves (base: start of a row, voff: lane offset in bytes)
  __device__ __forceinline__ char *row_base(long row) const { return reinterpret_cast<char *>(o + row * step); }
  __device__ __forceinline__ long step_bytes() const { return step * (long)sizeof(T); }
  __device__ __forceinline__ void store(char *base, unsigned &voff, T v) const {
    asm volatile("" : "+v"(voff));  // keeps the 32 -> 64 bit extension next to the store, where it folds into the address mode
    *reinterpret_cast<T *>(base + voff) = v;
  }
};
// The same rows written with non-temporal stores: the block is read again only by the next launch, long after it has
// left the caches.  Used by the bf16 matrix-core kernels, whose short main loops leave the stores exposed (measured on
// the benchmark layers: split bf16 -1.5 %, plain bf16 -2.5 %); for the fp32 / fp64 kernels it is within +-1 % either way
// and the first-layer kernels, which do nothing but store, are 30 % slower with it: they keep plain stores.
template <typename T> struct StreamRows : PlainRows<T> {
  __device__ __forceinline__ void put(long row, T v) const { store(this->row_base(row), this->lane_bytes, v); }
  __device__ __forceinline__ void store(char *base, unsigned &voff, T v) const {
    asm volatile("" : "+v"(voff));
    __builtin_nontemporal_store(v, reinterpret_cast<T *>(base + voff));
  }
};
// Rows written back into the staged chunk in LDS, in place of the pre-activations they were computed from (the rule reads
// a row before it writes it; one thread owns a (point, feature) column, so this is only for a wavefront per point).  The
// caller then copies the finished chunk to global memory with 16-byte stores.
template <typename T> struct LdsRows {
  T *o;         // the point's first row in the chunk
  long step;    // row pitch of the chunk, elements
  mutable unsigned lane_bytes = 0;
  __device__ __forceinline__ void put(long row, T v) const { store(row_base(row), lane_bytes, v); }
  __device__ __forceinline__ char *row_base(long row) const { return reinterpret_cast<char *>(o + row * step); }
  __device__ __forceinline__ long step_bytes() const { return step * (long)sizeof(T); }
  __device__ __forceinline__ void store(char *base, unsigned &voff, T v) const { *reinterpret_cast<T *>(base + voff) = v; }
};
struct Bf16Rows {  // rows of bf16 (the block between the layers of a plain-bf16 handle)
  __bf16 *o;
  long step;
  mutable unsigned lane_bytes = 0;
  __device__ __forceinline__ void put(long row, float v) const { store(row_base(row), lane_bytes, v); }
  __device__ __forceinline__ char *row_base(long row) const { return reinterpret_cast<char *>(o + row * step); }
  __device__ __forceinline__ long step_bytes() const { return step * 2; }
  __device__ __forceinline__ void store(char *base, unsigned &voff, float v) const {
    asm volatile("" : "+v"(voff));
    __builtin_nontemporal_store((__bf16)v, reinterpret_cast<__bf16 *>(base + voff));
  }
};

// c: the pair's column in the staged C tile (row pitch CROW elements, rows = the point's coefficient rows).
//
// The sum over directions is always taken the same way: direction i (counted from 0) belongs to group i % 4, each
// group is summed in order of i, and the four group sums are combined as (g0 + g1) + (g2 + g3).  WPP wavefronts
// (1, 2 or 4) share a point: wavefront `sub` takes the groups sub, sub + WPP, ... and writes their per-direction rows;
// for WPP > 1 the group sums of the other wavefronts reach wavefront 0 through LDS (`red`: this pair's first slot, slot
// stride 64 elements, kRedSlots(WPP) slots per point) and wavefront 0
// writes the collapsed row.  The result is therefore bit-identical for every WPP, i.e. for every tile shape.
// With WPP > 1 every thread of the workgroup must make the call (it holds a barrier); threads without a valid
// pair pass active = false.  Un-collapsed (standard) mode has no sum and is only built for WPP = 1.
// STD = false compiles the un-collapsed branch out (callers that are never launched in that mode).
template <typename T, typename Out, int WPP = 1, bool STD = true>
__device__ __forceinline__ void jet_rule(const T *c, int CROW, T bias, const Out &out, const LayerArgs<T> &a, bool active = true,
                                         int sub = 0, T *red = nullptr) {
  constexpr int NG = 4 / WPP;  // groups per wavefront
  const int R = a.R;
  T t = T(0), d1 = T(0), d2 = T(0);
  if (active) {
    const T z0 = c[0] + bias;
    act_eval<T>(a.act, z0, t, d1);
    d2 = act_d2<T>(a.act, t, d1);
    if (sub == 0) out.put(0, t);
  }
  if (STD && a.standard) {
    // un-collapsed ("standard") Taylor mode, kept for comparison: every direction carries its own
    // highest-order row (1 + K*R rows per point) and the sum over directions is taken after the last layer
    if (!active) return;
    if (a.order == 2) {  // rows 1..R first order, R+1..2R second order
      for (int r = 0; r < R; ++r) {
        const T z1 = c[(long)(1 + r) * CROW], z2 = c[(long)(1 + R + r) * CROW];
        const T h2 = d1 * z2 + d2 * z1 * z1;
        if (a.last) {
          out.put(1 + r, h2);
        } else {
          out.put(1 + r, d1 * z1);
          out.put(1 + R + r, h2);
        }
      }
    } else {  // rows 1+4r .. 4+4r: orders 1..4 of direction r
      const T d3 = act_d3<T>(a.act, t, d1), d4 = act_d4<T>(a.act, t, d1);
      for (int r = 0; r < R; ++r) {
        const T *cr = c + (long)(1 + 4 * r) * CROW;
        const T z1 = cr[0], z2 = cr[CROW], z3 = cr[2 * CROW], z4 = cr[3 * CROW];
        const T z1s = z1 * z1;
        const T h4 = d4 * z1s * z1s + T(6) * d3 * z1s * z2 + T(4) * d2 * z1 * z3 + T(3) * d2 * z2 * z2 + d1 * z4;
        if (a.last) {
          out.put(1 + r, h4);
        } else {
          const long row = 1 + 4 * r;
          out.put(row, d1 * z1);
          out.put(row + 1, d2 * z1s + d1 * z2);
          out.put(row + 2, d3 * z1s * z1 + T(3) * d2 * z1 * z2 + d1 * z3);
          out.put(row + 3, h4);
        }
      }
    }
    return;
  }
  T sg[NG];
#pragma unroll
  for (int k = 0; k < NG; ++k) sg[k] = T(0);
  T d3 = T(0), d4 = T(0);
  if (a.order == 2) {
    if (active) {
      int i0 = 0;
      if (a.last) {
        for (; i0 + 3 < R; i0 += 4) {  // NG independent LDS reads in flight per trip
          T z1[NG];
#pragma unroll
          for (int k = 0; k < NG; ++k) z1[k] = c[(1 + i0 + sub + k * WPP) * CROW];
#pragma unroll
          for (int k = 0; k < NG; ++k) sg[k] += z1[k] * z1[k];
        }
      } else {
        // one row address per trip (scalar when `out.o` is wavefront-uniform) and one constant lane offset per group:
        // the loop body is 2 LDS reads, 2 vector-ALU instructions and 1 store per direction plus a handful of scalar ones
        unsigned voff[NG];
#pragma unroll
        for (int k = 0; k < NG; ++k) voff[k] = out.lane_bytes + (unsigned)((sub + k * WPP) * out.step_bytes());
        char *rb = out.row_base(1);
        const long bump = 4 * out.step_bytes();
        const T *cr = c + CROW;
        // eight directions per trip while they last (their LDS reads are in flight together: the rule is bound by LDS
        // latency where few wavefronts share a SIMD), then four; a group still adds its directions in ascending order
        for (; i0 + 7 < R; i0 += 8, rb += 2 * bump, cr += 8 * CROW) {
          T z1[NG], y1[NG];
#pragma unroll
          for (int k = 0; k < NG; ++k) z1[k] = cr[(sub + k * WPP) * CROW];
#pragma unroll
          for (int k = 0; k < NG; ++k) y1[k] = cr[(4 + sub + k * WPP) * CROW];
#pragma unroll
          for (int k = 0; k < NG; ++k) {
            sg[k] += z1[k] * z1[k];
            out.store(rb, voff[k], d1 * z1[k]);
          }
#pragma unroll
          for (int k = 0; k < NG; ++k) {
            sg[k] += y1[k] * y1[k];
            out.store(rb + bump, voff[k], d1 * y1[k]);
          }
        }
        for (; i0 + 3 < R; i0 += 4, rb += bump, cr += 4 * CROW) {
          T z1[NG];
#pragma unroll
          for (int k = 0; k < NG; ++k) z1[k] = cr[(sub + k * WPP) * CROW];
#pragma unroll
          for (int k = 0; k < NG; ++k) {
            sg[k] += z1[k] * z1[k];
            out.store(rb, voff[k], d1 * z1[k]);
          }
        }
      }
#pragma unroll
      for (int k = 0; k < NG; ++k) {
        const int i = i0 + sub + k * WPP;
        if (i < R) {
          const T z1 = c[(long)(1 + i) * CROW];
          sg[k] += z1 * z1;
          if (!a.last) out.put(1 + i, d1 * z1);
        }
      }
    }
  } else if (active) {
    d3 = act_d3<T>(a.act, t, d1);
    d4 = act_d4<T>(a.act, t, d1);
    for (int i0 = 0; i0 < R; i0 += 4) {
#pragma unroll
      for (int k = 0; k < NG; ++k) {
        const int i = i0 + sub + k * WPP;
        if (i < R) {
          const T *cr = c + (long)(1 + 3 * i) * CROW;
          const T z1 = cr[0], z2 = cr[CROW], z3 = cr[2 * CROW];
          const T z1s = z1 * z1;
          sg[k] += d4 * z1s * z1s + T(6) * d3 * z1s * z2 + T(4) * d2 * z1 * z3 + T(3) * d2 * z2 * z2;
          if (!a.last) {
            const long row = 1 + 3 * i;
            out.put(row, d1 * z1);
            out.put(row + 1, d2 * z1s + d1 * z2);
            out.put(row + 2, d3 * z1s * z1 + T(3) * d2 * z1 * z2 + d1 * z3);
          }
        }
      }
    }
  }
  T s;
  if constexpr (WPP == 1) {
    if (!active) return;
    s = (sg[0] + sg[1]) + (sg[2] + sg[3]);
  } else {
    // wavefronts 1 .. WPP-1 hand their group sums to wavefront 0: slot (group - 1) / 2 for WPP = 2 (groups 1, 3),
    // slot group - 1 for WPP = 4 (groups 1, 2, 3)
    if (sub != 0) {
#pragma unroll
      for (int k = 0; k < NG; ++k) red[(WPP == 2 ? k : sub - 1) * 64] = sg[k];
    }
    __syncthreads();
    if (!active || sub != 0) return;
    if constexpr (WPP == 2) s = (sg[0] + red[0]) + (sg[1] + red[64]);
    else s = (sg[0] + red[0]) + (red[64] + red[128]);
  }
  if (a.order == 2) {
    const T z2 = c[(long)(R + 1) * CROW];
    out.put(a.last ? 1 : R + 1, d1 * z2 + d2 * s);
  } else {
    const T z4 = c[(long)(3 * R + 1) * CROW];
    out.put(a.last ? 1 : 3 * R + 1, d1 * z4 + s);
  }
}

// o: the pair's column in an output block of plain rows (row pitch ostep elements).
template <typename T>
__device__ __forceinline__ void jet_rule(const T *c, int CROW, T bias, T *o, long ostep, const LayerArgs<T> &a) {
  jet_rule<T, PlainRows<T>, 1>(c, CROW, bias, PlainRows<T>{o, ostep, 0u}, a);
}

// Element at byte offset `voff` (the lane's column) of a row whose start `row` is the same for the whole wavefront:
// the address is a scalar base plus a 32-bit lane offset, i.e. no vector-ALU address arithmetic.
template <typename T> __device__ __forceinline__ T lane_load(const T *row, unsigned &voff) {
  asm volatile("" : "+v"(voff));  // see PlainRows::store
  return *reinterpret_cast<const T *>(reinterpret_cast<const char *>(row) + voff);
}
template <typename T> __device__ __forceinline__ void lane_store(T *row, unsigned &voff, T v) {
  asm volatile("" : "+v"(voff));
  *reinterpret_cast<T *>(reinterpret_cast<char *>(row) + voff) = v;
}

// Record the pre-activation rows of one (point, feature) pair (bias on the order-0 row only).  zo: the point's row 0
// at the wavefront's first column (wavefront-uniform), voff: the lane's column in bytes.
template <typename T>
__device__ __forceinline__ void save_preactivations(const T *c, int CROW, T bias, T *zo, long zstep, unsigned voff, int rho) {
  lane_store<T>(zo, voff, c[0] + bias);
  for (int r = 1; r < rho; ++r) lane_store<T>(zo + r * zstep, voff, c[r * CROW]);
}

// Reverse of the collapsed rule for one (point, feature) pair.  z are the recorded pre-activations, hb the
// cotangents of the rule's outputs; d1 .. d5 depend on z_0 with d(d_k)/dz_0 = d_{k+1}.
// Order 2 (h_0 = t, h_{1,r} = d1 z_{1,r}, h_2 = d1 z_2 + d2 sum_r z_{1,r}^2):
//   zb_2     = d1 hb_2
//   zb_{1,r} = d1 hb_{1,r} + 2 d2 z_{1,r} hb_2
//   zb_0     = d1 hb_0 + d2 (sum_r hb_{1,r} z_{1,r} + hb_2 z_2) + d3 hb_2 sum_r z_{1,r}^2
// Order 4 (h_{1..3,r} and the collapsed h_4 as in jet_rule; z1, z2, z3 stand for z_{1,r}, z_{2,r}, z_{3,r}):
//   zb_4     = d1 hb_4
//   zb_{3,r} = d1 hb_3 + 4 d2 z1 hb_4
//   zb_{2,r} = d1 hb_2 + 3 d2 z1 hb_3 + 6 (d3 z1^2 + d2 z2) hb_4
//   zb_{1,r} = d1 hb_1 + 2 d2 z1 hb_2 + 3 (d3 z1^2 + d2 z2) hb_3 + 4 (d4 z1^3 + 3 d3 z1 z2 + d2 z3) hb_4
//   zb_0     = d1 hb_0 + sum_r [ d2 z1 hb_1 + (d3 z1^2 + d2 z2) hb_2 + (d4 z1^3 + 3 d3 z1 z2 + d2 z3) hb_3 ]
//              + hb_4 [ d2 z_4 + sum_r (d5 z1^4 + 6 d4 z1^2 z2 + 4 d3 z1 z3 + 3 d3 z2^2) ]
// c: cotangent column in the staged C tile; zs / o: the point's row 0 of the recorded block / of the output block at the
// wavefront's first column (wavefront-uniform); voff: the lane's column in bytes.
template <typename T>
__device__ __forceinline__ void jet_rule_bwd(const T *c, int CROW, const T *zs, long zstep, T *o, long ostep, unsigned voff,
                                             const LayerArgs<T> &a) {
  const int R = a.R;
  const T z0 = lane_load<T>(zs, voff);
  T t, d1;
  act_eval<T>(a.act, z0, t, d1);
  const T d2 = act_d2<T>(a.act, t, d1), d3 = act_d3<T>(a.act, t, d1);
  if (a.order == 2) {
    const T hb0 = c[0], hb2 = c[(R + 1) * CROW];
    const T z2 = lane_load<T>(zs + (R + 1) * zstep, voff);
    const T w = T(2) * d2 * hb2;
    // four directions per trip, their loads issued together (the recorded rows come from HBM / L2); the two sums are
    // kept in four interleaved groups and combined as (g0 + g1) + (g2 + g3)
    T sg[4] = {T(0), T(0), T(0), T(0)}, dg[4] = {T(0), T(0), T(0), T(0)};
    int r = 1;
    for (; r + 3 <= R; r += 4) {
      T z1[4], hb1[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) z1[k] = lane_load<T>(zs + (r + k) * zstep, voff);
#pragma unroll
      for (int k = 0; k < 4; ++k) hb1[k] = c[(r + k) * CROW];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        sg[k] += z1[k] * z1[k];
        dg[k] += hb1[k] * z1[k];
        lane_store<T>(o + (r + k) * ostep, voff, d1 * hb1[k] + w * z1[k]);
      }
    }
    for (int k = 0; r <= R; ++r, ++k) {
      const T z1 = lane_load<T>(zs + r * zstep, voff), hb1 = c[r * CROW];
      sg[k] += z1 * z1;
      dg[k] += hb1 * z1;
      lane_store<T>(o + r * ostep, voff, d1 * hb1 + w * z1);
    }
    const T s = (sg[0] + sg[1]) + (sg[2] + sg[3]), dot = (dg[0] + dg[1]) + (dg[2] + dg[3]);
    lane_store<T>(o + (R + 1) * ostep, voff, d1 * hb2);
    lane_store<T>(o, voff, d1 * hb0 + d2 * (dot + hb2 * z2) + d3 * s * hb2);
  } else {
    const T d4 = act_d4<T>(a.act, t, d1), d5 = act_d5<T>(a.act, t, d1);
    const T hb0 = c[0], hb4 = c[(3 * R + 1) * CROW];
    const T z4 = lane_load<T>(zs + (3 * R + 1) * zstep, voff);
    T acc = T(0), s4 = T(0);
    for (int r = 0; r < R; ++r) {
      const T *zr = zs + (1 + 3 * r) * zstep;
      const T *cr = c + (1 + 3 * r) * CROW;
      T *orow = o + (1 + 3 * r) * ostep;
      const T z1 = lane_load<T>(zr, voff), z2 = lane_load<T>(zr + zstep, voff), z3 = lane_load<T>(zr + 2 * zstep, voff);
      const T hb1 = cr[0], hb2 = cr[CROW], hb3 = cr[2 * CROW];
      const T z1s = z1 * z1;
      const T p2 = d3 * z1s + d2 * z2;                              // d h_2 / d z_0
      const T p3 = d4 * z1s * z1 + T(3) * d3 * z1 * z2 + d2 * z3;   // d h_3 / d z_0
      lane_store<T>(orow, voff, d1 * hb1 + T(2) * d2 * z1 * hb2 + T(3) * p2 * hb3 + T(4) * p3 * hb4);
      lane_store<T>(orow + ostep, voff, d1 * hb2 + T(3) * d2 * z1 * hb3 + T(6) * p2 * hb4);
      lane_store<T>(orow + 2 * ostep, voff, d1 * hb3 + T(4) * d2 * z1 * hb4);
      acc += d2 * z1 * hb1 + p2 * hb2 + p3 * hb3;
      s4 += d5 * z1s * z1s + T(6) * d4 * z1s * z2 + T(4) * d3 * z1 * z3 + T(3) * d3 * z2 * z2;
    }
    lane_store<T>(o + (3 * R + 1) * ostep, voff, d1 * hb4);
    lane_store<T>(o, voff, d1 * hb0 + acc + hb4 * (d2 * z4 + s4));
  }
}

}  // namespace ctm
