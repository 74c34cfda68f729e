// Dense combination on compacted rows with fp32 MFMA (v_mfma_f32_32x32x2_f32), fused with the
// gather of the input rows, bias, activation and the compare-and-emit step (a row is reported
// as changed only if its new value differs bitwise from the cached one; Sec. 2.5.2).
//
// Every output element is one chain of fused multiply-adds over k = 0 .. K-1 in ascending order
// starting from +0 (the MFMA unit applies its two k-steps in that order), independent of the
// tile or row slot it is computed in, so a row's result never depends on which other rows share
// the launch.  Zero-padded k-steps leave the accumulator unchanged.
#include "ctx.h"

namespace ink {

typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int KT = 32;       // k-chunk staged in LDS

__device__ __forceinline__ float agg_value(const XformArgs &x, int64_t row, int k) {
  float a = x.A[row * x.lda + k];
  if (x.mean_deg) { int dg = x.mean_deg[row]; a = __fdiv_rn(a, (float)(dg > 0 ? dg : 1)); }
  return a;
}

template <int MODE>
__device__ __forceinline__ float fetch_x(const XformArgs &x, int64_t row, int k) {
  if (MODE == 0) {           // SAGE: [alpha | h_prev]
    if (k < x.d_in) return agg_value(x, row, k);
    if (k < 2 * x.d_in) return x.Hp[row * x.ldh + (k - x.d_in)];
    return 0.f;
  } else if (MODE == 1) {    // GIN: (1 + eps) h_prev + alpha
    if (k < x.d_in) return __fadd_rn(__fmul_rn(1.0f + x.eps, x.Hp[row * x.ldh + k]), agg_value(x, row, k));
    return 0.f;
  } else if (MODE == 3) {    // GCN: h = act(c_v (S + own scaled message) + b); also stored as h_l
    if (k >= x.d_in) return 0.f;
    float v = __fmul_rn(x.cnorm[row], __fadd_rn(x.A[row * x.lda + k], x.Hp[row * x.ldh + k]));
    if (x.in_bias) v = __fadd_rn(v, x.in_bias[k]);
    if (x.in_user) v = __fadd_rn(v, x.in_user[row * x.ld_in_user + k]);
    if (x.in_relu) v = v > 0.f ? v : 0.f;
    if (x.h_store) x.h_store[row * x.ld_hs + k] = v;
    return v;
  } else {                   // dense rows
    if (k < x.d_in) return x.Hp[row * x.ldh + k];
    return 0.f;
  }
}

__device__ __forceinline__ void ld4v(const float *p, float out[4]) {
  float4 v = *reinterpret_cast<const float4 *>(p);
  out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}

// four consecutive inputs k .. k + 3 (k a multiple of 4) of one row; 16-byte loads when the group
// lies inside one table row, element-wise otherwise.  Results are identical to fetch_x.
template <int MODE>
__device__ __forceinline__ void fetch_x4(const XformArgs &x, int64_t row, int k, float out[4]) {
  if (MODE == 0) {
    if ((x.d_in & 3) == 0 && k + 3 < 2 * x.d_in) {
      if (k < x.d_in) {
        ld4v(x.A + row * x.lda + k, out);
        if (x.mean_deg) {
          int dg = x.mean_deg[row];
          float dv = (float)(dg > 0 ? dg : 1);
#pragma unroll
          for (int i = 0; i < 4; i++) out[i] = __fdiv_rn(out[i], dv);
        }
      } else {
        ld4v(x.Hp + row * x.ldh + (k - x.d_in), out);
      }
      return;
    }
  } else if (MODE == 1) {
    if (k + 3 < x.lda && k + 3 < x.ldh) {
      float a[4], h[4];
      ld4v(x.A + row * x.lda + k, a);
      ld4v(x.Hp + row * x.ldh + k, h);
      float dv = 1.f;
      if (x.mean_deg) { int dg = x.mean_deg[row]; dv = (float)(dg > 0 ? dg : 1); }
#pragma unroll
      for (int i = 0; i < 4; i++) {
        float av = x.mean_deg ? __fdiv_rn(a[i], dv) : a[i];
        out[i] = k + i < x.d_in ? __fadd_rn(__fmul_rn(1.0f + x.eps, h[i]), av) : 0.f;
      }
      return;
    }
  } else if (MODE == 3) {
    if (k + 3 < x.lda && k + 3 < x.ldh && !x.in_user) {      // rows with a user term take the element-wise path
      float a[4], h[4];
      ld4v(x.A + row * x.lda + k, a);
      ld4v(x.Hp + row * x.ldh + k, h);
      float cv = x.cnorm[row];
      float b[4] = {0.f, 0.f, 0.f, 0.f};
      if (x.in_bias) {       // one 16-byte load when the group lies inside the bias vector
        if (k + 3 < x.d_in) ld4v(x.in_bias + k, b);
        else
#pragma unroll
          for (int i = 0; i < 4; i++) if (k + i < x.d_in) b[i] = x.in_bias[k + i];
      }
#pragma unroll
      for (int i = 0; i < 4; i++) {
        float v = __fmul_rn(cv, __fadd_rn(a[i], h[i]));
        if (x.in_bias && k + i < x.d_in) v = __fadd_rn(v, b[i]);
        if (x.in_relu) v = v > 0.f ? v : 0.f;
        out[i] = k + i < x.d_in ? v : 0.f;
      }
      if (x.h_store && k + 3 < x.ld_hs)
        *reinterpret_cast<float4 *>(x.h_store + row * x.ld_hs + k) = make_float4(out[0], out[1], out[2], out[3]);
      return;
    }
  } else {
    if ((x.ldh & 3) == 0 && k + 3 < x.ldh) {
      ld4v(x.Hp + row * x.ldh + k, out);
#pragma unroll
      for (int i = 0; i < 4; i++) out[i] = k + i < x.d_in ? out[i] : 0.f;
      return;
    }
  }
#pragma unroll
  for (int i = 0; i < 4; i++) out[i] = fetch_x<MODE>(x, row, k + i);
}

// LDS layouts (floats): X tile [BM][2][16] with row stride XS, W tile [Np][2][16] with row stride
// XS.  Index [.][p][s] holds k = k0 + 2 s + p, so the 16 values a lane feeds to the 16 MFMA steps
// of a chunk (lanes 0-31 take the even k, lanes 32-63 the odd k) are contiguous: four 16-byte LDS
// reads.  The stride of 36 floats spreads 16 lanes x 4 banks over all 64 banks.  The weights are
// stored in global memory already in this order (see xform_weight_index).
constexpr int XS = 36;

// Compute phase of one k-chunk for the NTW column tiles ct0, ct0 + 2, ... of this wave: all LDS
// reads of a tile are issued before its 16 back-to-back MFMAs.
template <int NTW, int CS>
__device__ __forceinline__ void mfma_chunk(const float *Xs, const float *Ws, int rt, int ct0, int l, f16v *acc) {
  const float *ap = Xs + (rt * 32 + (l & 31)) * XS + (l >> 5) * 16;
  float a[16];
#pragma unroll
  for (int v = 0; v < 4; v++) {
    float4 t4 = *reinterpret_cast<const float4 *>(ap + 4 * v);
    a[4 * v] = t4.x; a[4 * v + 1] = t4.y; a[4 * v + 2] = t4.z; a[4 * v + 3] = t4.w;
  }
#pragma unroll
  for (int i = 0; i < NTW; i++) {
    const float *bp = Ws + ((ct0 + CS * i) * 32 + (l & 31)) * XS + (l >> 5) * 16;
    float b[16];
#pragma unroll
    for (int v = 0; v < 4; v++) {
      float4 t4 = *reinterpret_cast<const float4 *>(bp + 4 * v);
      b[4 * v] = t4.x; b[4 * v + 1] = t4.y; b[4 * v + 2] = t4.z; b[4 * v + 3] = t4.w;
    }
#pragma unroll
    for (int sidx = 0; sidx < 16; sidx++)
      acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[sidx], b[sidx], acc[i], 0, 0, 0);
  }
}

// Epilogue of a workgroup's tile: bias, user term, output scale, activation, then either a plain
// store or compare-and-emit against the cached table row.  A lane holds rows
// 8*(r/4) + 4*(l/32) + r%4 of its row tile, column l % 32 of each of its column tiles.
template <int TPW, int CS, int NT, int BM>
__device__ __forceinline__ void xform_epilogue(const XformArgs &x, const f16v *acc, const int64_t *srow, const int64_t *sout,
                                               int *schg, int rt, int ct0, int l, int t, int64_t r0) {
#pragma unroll
  for (int i = 0; i < TPW; i++) {
    int ct = ct0 + CS * i;
    if (ct >= NT) continue;
    int col = ct * 32 + (l & 31);
    if (col >= x.n_out) continue;
    float bias = x.bias ? x.bias[col] : 0.f;
    float oldv[16];
    if (x.to_table) {      // all loads of the cached values first, then compare and store
#pragma unroll
      for (int r = 0; r < 16; r++) {
        int rl = rt * 32 + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
        oldv[r] = srow[rl] >= 0 ? x.out[sout[rl] * x.ld_out + col] : 0.f;
      }
    }
#pragma unroll
    for (int r = 0; r < 16; r++) {
      int rl = rt * 32 + 8 * (r >> 2) + 4 * (l >> 5) + (r & 3);
      int64_t row = srow[rl];
      if (row < 0) continue;
      float v = acc[i][r];
      if (x.bias) v = __fadd_rn(v, bias);
      if (x.user) v = __fadd_rn(v, x.user[sout[rl] * x.ld_user + col]);
      if (x.out_scale) v = __fmul_rn(v, x.out_scale[sout[rl]]);
      if (x.relu) v = v > 0.f ? v : 0.f;
      int64_t j = r0 + rl;
      if (x.to_table) {
        float old = oldv[r];
        if (x.old_rows) x.old_rows[j * x.ld_old + col] = old;
        if (__float_as_uint(old) != __float_as_uint(v)) { x.out[sout[rl] * x.ld_out + col] = v; schg[rl] = 1; }
      } else {
        x.out[j * x.ld_out + col] = v;
      }
    }
  }
  if (x.to_table && x.row_changed) {
    __syncthreads();
    if (t < BM && srow[t] >= 0) x.row_changed[r0 + t] = (uint8_t)schg[t];
  }
}

// BM = rows per workgroup (64 or 128), NT = number of 32-column tiles (Np / 32), NW = waves per
// workgroup.  With RT = BM / 32 row tiles, wave w works on row tile w % RT and on the column tiles
// w / RT, w / RT + NW / RT, ...
template <int MODE, int NT, int NW, int BM>
__global__ __launch_bounds__(NW * 64) void k_xform(XformArgs x) {
  extern __shared__ float smem[];
  float *Xs = smem;                           // [BM][XS]
  float *Ws = smem + BM * XS;                 // [Np][XS]
  __shared__ int64_t srow[BM];     // input row (gather) of each tile row, -1 past the end
  __shared__ int64_t sout[BM];     // table row written by the epilogue
  __shared__ int schg[BM];
  constexpr int RT = BM / 32;
  constexpr int CS = NW / RT;                 // column-tile stride between the tiles of one wave
  constexpr int TPW = (NT + CS - 1) / CS;
  constexpr int Np = NT * 32;
  constexpr int NTHR = NW * 64;
  constexpr int KPT = KT * BM / NTHR >= 4 ? KT * BM / NTHR : 4;   // consecutive k of one row that a thread stages (8 or 4)
  constexpr int XTHR = KT * BM / KPT;         // threads that stage X (all of them up to 8 waves)
  const int t = threadIdx.x, l = t & 63, w = t >> 6;
  const int rt = w % RT;                      // row tile of this wave
  const int ct0 = w / RT;                     // first column tile; then += CS
  const int64_t r0 = (int64_t)blockIdx.x * BM;
  int64_t n_rows = x.n_rows;
  if (x.n_rows_dev) {          // the launch covers an upper bound; workgroups past the count leave
    int64_t nd = *x.n_rows_dev;
    n_rows = nd < n_rows ? nd : n_rows;
    if (r0 >= n_rows) return;
  }
  if (t < BM) {
    int64_t j = r0 + t;
    int64_t row = -1;
    if (j < n_rows) row = (MODE == 2) ? j : (x.rows ? (int64_t)x.rows[j] : j);
    srow[t] = row;
    sout[t] = (row >= 0 && MODE == 2 && x.to_table && x.out_rows) ? (int64_t)x.out_rows[j] : row;
    schg[t] = 0;
  }
  f16v acc[TPW];
#pragma unroll
  for (int i = 0; i < TPW; i++)
#pragma unroll
    for (int r = 0; r < 16; r++) acc[i][r] = 0.f;
  __syncthreads();
  // thread -> row t / 4, 8 consecutive k of the X chunk; the next chunk's values are fetched into
  // registers before the MFMA phase so that the gather latency overlaps it
  const bool xstage = t < XTHR;
  const int xr = (t % XTHR) / (KT / KPT), xks = (t % (KT / KPT)) * KPT;
  const int64_t xrow = xstage ? srow[xr] : -1;
  float xv[KPT];
  auto fetch_chunk = [&](int k0) {
#pragma unroll
    for (int kk = 0; kk < KPT; kk++) xv[kk] = 0.f;
    if (xrow >= 0) {
#pragma unroll
      for (int kk = 0; kk < KPT; kk += 4) fetch_x4<MODE>(x, xrow, k0 + xks + kk, xv + kk);
    }
  };
  // GCN rows whose width is a multiple of the chunk: the loads of the next chunk are issued a
  // whole iteration before their values are scaled, biased, stored as h and staged, so the
  // gather latency overlaps the barriers, the weight staging and the MFMAs of the chunk between
  const bool raw3 = MODE == 3 && x.d_in == x.Kp && x.lda >= x.Kp && x.ldh >= x.Kp && (!x.h_store || x.ld_hs >= x.Kp) && !x.in_user;
  float ra[KPT], rh[KPT], rb[KPT];
  const float cv3 = (raw3 && xrow >= 0) ? x.cnorm[xrow] : 0.f;
  auto issue3 = [&](int k0) {
    if (xrow < 0) return;
#pragma unroll
    for (int kk = 0; kk < KPT; kk += 4) {
      int k = k0 + xks + kk;
      ld4v(x.A + xrow * x.lda + k, ra + kk);
      ld4v(x.Hp + xrow * x.ldh + k, rh + kk);
      if (x.in_bias) ld4v(x.in_bias + k, rb + kk);
    }
  };
  auto finish3 = [&](int k0) {
#pragma unroll
    for (int kk = 0; kk < KPT; kk++) xv[kk] = 0.f;
    if (xrow < 0) return;
#pragma unroll
    for (int kk = 0; kk < KPT; kk++) {
      float v = __fmul_rn(cv3, __fadd_rn(ra[kk], rh[kk]));
      if (x.in_bias) v = __fadd_rn(v, rb[kk]);
      if (x.in_relu) v = v > 0.f ? v : 0.f;
      xv[kk] = v;
    }
    if (x.h_store) {
#pragma unroll
      for (int kk = 0; kk < KPT; kk += 4)
        *reinterpret_cast<float4 *>(x.h_store + xrow * x.ld_hs + k0 + xks + kk) = make_float4(xv[kk], xv[kk + 1], xv[kk + 2], xv[kk + 3]);
    }
  };
  if (raw3) issue3(0); else fetch_chunk(0);
  for (int k0 = 0; k0 < x.Kp; k0 += KT) {
    if (raw3) finish3(k0);
    if (xstage) {   // even k first, then odd k
      float *xp = Xs + xr * XS + (xks >> 1);
      if constexpr (KPT == 8) {
        *reinterpret_cast<float4 *>(xp) = make_float4(xv[0], xv[2], xv[4], xv[6]);
        *reinterpret_cast<float4 *>(xp + 16) = make_float4(xv[1], xv[3], xv[5], xv[7]);
      } else {
        *reinterpret_cast<float2 *>(xp) = make_float2(xv[0], xv[2]);
        *reinterpret_cast<float2 *>(xp + 16) = make_float2(xv[1], xv[3]);
      }
    }
    {   // stage the W chunk: global [Np][32] in LDS order -> rows of stride XS
      const float4 *src = reinterpret_cast<const float4 *>(x.W + (int64_t)k0 * Np);
      constexpr int n4 = KT * Np / 4;
#pragma unroll
      for (int i = t; i < n4; i += NTHR) *reinterpret_cast<float4 *>(Ws + (i >> 3) * XS + (i & 7) * 4) = src[i];
    }
    if (raw3 && k0 + KT < x.Kp) issue3(k0 + KT);
    __syncthreads();
    if (!raw3 && k0 + KT < x.Kp) fetch_chunk(k0 + KT);
    // this wave owns TPW column tiles, or one fewer when the last one would lie past NT
    if (ct0 + (TPW - 1) * CS < NT) mfma_chunk<TPW, CS>(Xs, Ws, rt, ct0, l, acc);
    else if (TPW > 1) mfma_chunk<(TPW > 1 ? TPW - 1 : 1), CS>(Xs, Ws, rt, ct0, l, acc);
    __syncthreads();
  }
  xform_epilogue<TPW, CS, NT, BM>(x, acc, srow, sout, schg, rt, ct0, l, t, r0);
}

#ifndef INK_XF_WIDE_FROM
#define INK_XF_WIDE_FROM 3      // 8 waves per workgroup from this many column tiles on
#endif
#ifndef INK_XF_WIDER_FROM
#define INK_XF_WIDER_FROM 5     // 16 waves per workgroup from this many column tiles on
#endif

// 64 rows per workgroup: 128 rows (half the weight staging per row) measured the same or slower
template <int MODE, int NT>
static void launch_nt(ink_ctx *c, const XformArgs &x) {
  constexpr int BM = 64;
  size_t sh = (size_t)(BM + x.Np) * XS * sizeof(float);
  dim3 grid((unsigned)((x.n_rows + BM - 1) / BM));
  if constexpr (NT >= INK_XF_WIDER_FROM) hipLaunchKernelGGL((k_xform<MODE, NT, 16, BM>), grid, dim3(1024), sh, c->stream, x);
  else if constexpr (NT >= INK_XF_WIDE_FROM) hipLaunchKernelGGL((k_xform<MODE, NT, 8, BM>), grid, dim3(512), sh, c->stream, x);
  else hipLaunchKernelGGL((k_xform<MODE, NT, 4, BM>), grid, dim3(256), sh, c->stream, x);
}

template <int MODE>
static hipError_t launch(ink_ctx *c, const XformArgs &x) {
  switch (x.Np / 32) {
    case 1: launch_nt<MODE, 1>(c, x); break;
    case 2: launch_nt<MODE, 2>(c, x); break;
    case 3: launch_nt<MODE, 3>(c, x); break;
    case 4: launch_nt<MODE, 4>(c, x); break;
    case 5: launch_nt<MODE, 5>(c, x); break;
    case 6: launch_nt<MODE, 6>(c, x); break;
    case 7: launch_nt<MODE, 7>(c, x); break;
    case 8: launch_nt<MODE, 8>(c, x); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t xform_run(ink_ctx *c, const XformArgs &x) {
  if (x.n_rows <= 0) return hipSuccess;
  if (x.Np % 32 || x.Kp % KT || x.Np > 256) return hipErrorInvalidValue;
  switch (x.mode) {
    case 0: return launch<0>(c, x);
    case 1: return launch<1>(c, x);
    case 2: return launch<2>(c, x);
    case 3: return launch<3>(c, x);
  }
  return hipErrorInvalidValue;
}

}  // namespace ink
