// Partial query projection (Section 4.3 "Decoding Stage": attention input of the previous layer
// times the partial query weight) and the small finalisation step (bias, rotary embedding and the
// partial skew A_h[:, idx_h] for models whose skew cannot be folded into W_Q).
//
// The projection reads the weight once (it is weight-read bound: B is 4..20 rows).  For half
// precision it runs on the matrix cores: the weight blob is stored in MFMA fragment order, so that
// every wave-wide load is one contiguous 1 KiB piece, the batch rows are the N side of a
// 16x16x32 MFMA, and K is split across waves to get enough waves in flight; the split-K partial
// sums are written out and added, in a fixed order, by the consumer.  float32 (and half with
// D % 32 != 0) uses a plain FMA kernel over the same split.
#include "ig_internal.h"

ProjGeom ig_proj_geom(const ig_desc *d) {
  ProjGeom g;
  const int D = d->H * d->d;
  g.C = d->rope ? D : d->H * d->r;
  g.nCblk = (g.C + 15) / 16;
  g.Cpad = g.nCblk * 16;
  g.NBtot = (d->B + 15) / 16;
  g.Bpad = g.NBtot * 16;
  g.mfma = d->dtype == IG_F16 && D % 32 == 0;
  const int units = g.mfma ? D / 32 : D;          // K units that can be split
  g.nKblk = g.mfma ? D / 32 : 0;
  // aim for >= 4096 waves (16 per compute unit: a wave then has a single batch of K blocks; measured
  // on a 4096 x 4096 weight, 8.8 -> 7.6 us against 2048 waves) but never more than IG_KS_MAX partial sums
  const int col_waves = g.mfma ? g.nCblk : (g.Cpad + 63) / 64;
  int ks = (4096 + col_waves - 1) / col_waves;
  if (ks > IG_KS_MAX) ks = IG_KS_MAX;
  if (ks > units) ks = units;
  if (ks < 1) ks = 1;
  g.kb_per = (units + ks - 1) / ks;
  g.KS = (units + g.kb_per - 1) / g.kb_per;
  return g;
}

namespace {

// ---- weight blob construction -------------------------------------------------------------------
// Column c of the blob is column colmap(c) of Wq: h*d + idx[h*r + j] for c = h*r + j (folded), or c
// itself (rope: every column kept).
__device__ __forceinline__ int colmap(int c, int d, int r, const int32_t *idx) {
  if (!idx) return c;
  int h = c / r, j = c % r;
  return h * d + min(max(idx[h * r + j], 0), d - 1);   // an index outside the head is clamped
}

// MFMA fragment order: piece (cblk, kblk) is 64 lanes x 8 halves; lane (kg = lane/16, i = lane%16)
// holds W[k = kblk*32 + kg*8 + e][col(cblk*16 + i)], e < 8.
__global__ void wq_build_mfma(const half_t *W, const int32_t *idx, half8 *blob, int D, int d, int r,
                              int C, int nCblk, int nKblk) {
  long g = (long)blockIdx.x * blockDim.x + threadIdx.x;
  long total = (long)nCblk * nKblk * 64;
  if (g >= total) return;
  int lane = g & 63;
  long piece = g >> 6;
  int kblk = piece % nKblk, cblk = piece / nKblk;
  int i = lane & 15, kg = lane >> 4;
  int c = cblk * 16 + i;
  half8 v;
  if (c < C) {
    int col = colmap(c, d, r, idx);
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = W[(long)(kblk * 32 + kg * 8 + e) * D + col];
  } else {
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (half_t)0;
  }
  blob[g] = v;
}

// Plain layout for the FMA kernel: blob[k][c], c < Cpad (zero padded).
template <typename T>
__global__ void wq_build_plain(const T *W, const int32_t *idx, T *blob, int D, int d, int r, int C,
                               int Cpad) {
  long g = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= (long)D * Cpad) return;
  int c = g % Cpad;
  long k = g / Cpad;
  blob[g] = (c < C) ? W[k * D + colmap(c, d, r, idx)] : (T)0;
}

// ---- projection ---------------------------------------------------------------------------------
// Wave (cblk, ks): part[ks][n][cblk*16 + i] = sum over its K blocks of W^T-fragment x x-fragment.
// A operand = weight piece (M side = 16 output columns), B operand = 16 batch rows of x.
// Result lane l, register v -> column cblk*16 + 4*(l/16) + v, batch row l%16.
template <int NB>
__global__ __launch_bounds__(256) void project_mfma(const half8 *__restrict__ blob,
                                                    const half_t *__restrict__ x,
                                                    float *__restrict__ part, int B, int D,
                                                    int nCblk, int nKblk, int kb_per, int KS,
                                                    int Bpad, int Cpad) {
  const int lane = threadIdx.x & 63;
  const long gw = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (gw >= (long)nCblk * KS) return;
  const int cblk = gw % nCblk, ks = gw / nCblk;
  const int nb0 = blockIdx.y * NB;
  const int n = lane & 15, kg = lane >> 4;
  const int kb0 = ks * kb_per, kb1 = min(nKblk, kb0 + kb_per);
  floatx4 acc[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
  const half8 *wp = blob + ((long)cblk * nKblk) * 64 + lane;
  const half8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
  // K blocks are taken KB at a time: all weight pieces and x fragments of a batch are loaded before
  // the first MFMA, so a wave keeps KB * (1 + NB) KiB in flight (a block past the end is clamped
  // to the last one and its MFMA skipped).
  constexpr int KB = NB == 1 ? 8 : (NB == 2 ? 6 : 4);
  for (int kb = kb0; kb < kb1; kb += KB) {
    half8 a[KB], bfrag[NB][KB];
#pragma unroll
    for (int t = 0; t < KB; ++t) {
      const int kbt = min(kb + t, kb1 - 1);
      a[t] = wp[(long)kbt * 64];
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int row = (nb0 + i) * 16 + n;
        bfrag[i][t] = zero;
        if (row < B) bfrag[i][t] = *reinterpret_cast<const half8 *>(x + (long)row * D + kbt * 32 + kg * 8);
      }
    }
#pragma unroll
    for (int t = 0; t < KB; ++t) {
      if (kb + t < kb1) {
#pragma unroll
        for (int i = 0; i < NB; ++i)
          acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[t], bfrag[i][t], acc[i], 0, 0, 0);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    int row = (nb0 + i) * 16 + n;
    if (row < Bpad) {
      float *o = part + ((long)ks * Bpad + row) * Cpad + cblk * 16 + kg * 4;
      *reinterpret_cast<floatx4 *>(o) = acc[i];
    }
  }
}

// The same product for more than 16 batch rows (NB blocks of 16) with the x fragments shared
// through LDS.  With NB = 2 the plain kernel above issues one weight load and two x loads per K
// block and needs three batches of loads per wave for the register budget; here the four waves of
// a workgroup (four neighbouring column blocks, the same K slice) stage the NB*16 rows of x for
// their K slice in LDS once, a wave keeps only its weight pieces in registers -- all of its K slice
// in flight at once, up to PKB pieces -- and reads each x fragment from LDS right before the MFMA
// that uses it.  grid (ceil(nCblk/4), KS); LDS row stride padded by 16 bytes so that the 16 rows a
// fragment read touches fall into different banks.
template <int NB, int PKB>
__global__ __launch_bounds__(256) void project_mfma_shared(const half8 *__restrict__ blob,
                                                           const half_t *__restrict__ x,
                                                           float *__restrict__ part, int B, int D,
                                                           int nCblk, int nKblk, int kb_per, int Bpad,
                                                           int Cpad) {
  extern __shared__ uint4 xs[];                       // [NB*16 rows][kb_per*4 + 1] 16-byte pieces
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int ks = blockIdx.y;
  const int cblk_raw = blockIdx.x * 4 + w;
  const bool live = cblk_raw < nCblk;                 // a surplus wave still helps staging x
  const int cblk = min(cblk_raw, nCblk - 1);
  const int n = lane & 15, kg = lane >> 4;
  const int kb0 = ks * kb_per, kb1 = min(nKblk, kb0 + kb_per);
  const int nkb = kb1 - kb0;
  // x rows of the slice (rows past B are zero): loaded first, because they are needed first -- a
  // wave's loads return in the order it issued them -- then the weight pieces of the whole K slice
  const int ppr = kb_per * 4, stride = ppr + 1;       // 16-byte pieces per row, padded stride
  const int pieces = NB * 16 * ppr;
  constexpr int XPT = NB * 16 * PKB * 4 / 256;         // x pieces per thread at most
  uint4 xv[XPT];
#pragma unroll
  for (int u = 0; u < XPT; ++u) {
    const int p = threadIdx.x + u * 256;
    const int row = p / ppr, c = p - row * ppr;
    xv[u] = make_uint4(0, 0, 0, 0);
    if (p < pieces && row < B && kb0 * 4 + c < nKblk * 4)
      xv[u] = *reinterpret_cast<const uint4 *>(x + (long)row * D + (long)kb0 * 32 + c * 8);
  }
  half8 a[PKB];
  const half8 *wp = blob + ((long)cblk * nKblk + kb0) * 64 + lane;
#pragma unroll
  for (int t = 0; t < PKB; ++t) a[t] = wp[(long)min(t, nkb - 1) * 64];
#pragma unroll
  for (int u = 0; u < XPT; ++u) {
    const int p = threadIdx.x + u * 256;
    const int row = p / ppr, c = p - row * ppr;
    if (p < pieces) xs[row * stride + c] = xv[u];
  }
  __syncthreads();
  if (!live) return;
  floatx4 acc[NB];
#pragma unroll
  for (int i = 0; i < NB; ++i) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int t = 0; t < PKB; ++t) {
    if (t < nkb) {
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const uint4 raw = xs[(i * 16 + n) * stride + t * 4 + kg];
        acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[t], *reinterpret_cast<const half8 *>(&raw), acc[i], 0, 0, 0);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    const int row = i * 16 + n;
    if (row < Bpad) {
      float *o = part + ((long)ks * Bpad + row) * Cpad + cblk * 16 + kg * 4;
      *reinterpret_cast<floatx4 *>(o) = acc[i];
    }
  }
}

// One thread per output column, 16 batch rows per pass, K rows [ks*kb_per, ...).
template <typename T>
__global__ __launch_bounds__(64) void project_fma(const T *__restrict__ blob, const T *__restrict__ x,
                                                  float *__restrict__ part, int B, int D, int kb_per,
                                                  int Bpad, int Cpad) {
  const int c = blockIdx.x * 64 + threadIdx.x;
  const int ks = blockIdx.y;
  const int n0 = blockIdx.z * 16;
  if (c >= Cpad) return;
  const int k0 = ks * kb_per, k1 = min(D, k0 + kb_per);
  float acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;
  for (int k = k0; k < k1; ++k) {
    float wv = (float)blob[(long)k * Cpad + c];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      int row = n0 + i;
      float xv = (row < B) ? (float)x[(long)row * D + k] : 0.f;
      acc[i] = fmaf(xv, wv, acc[i]);
    }
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) part[((long)ks * Bpad + n0 + i) * Cpad + c] = acc[i];
}

// ---- index-only partial weight ------------------------------------------------------------------
// Section 6.2 "Memory Consumption": instead of a second copy of the kept columns, only their
// indices are stored and the columns are taken from the full (skewed) query weight, which the
// model keeps on the GPU anyway.  Picking 2-byte columns out of a row-major matrix touches nearly
// every 64-byte line of it, so the kernel reads the rows of a head whole, with 16-byte loads, and
// multiplies all d columns (fp32 FMAs: B*D*D of them, below the time of the D*D read for B <= 16);
// the kept columns are picked from the result.
// Workgroup (h, ks, batch block): 4 waves; a wave-wide load covers 64/LPRp rows of the head's
// d-column span (LPR = 16-byte pieces per row, LPRp = LPR rounded up to a power of two).  The
// NBR batch rows of x for the K chunk are staged in LDS as float.  The sums over a wave's rows are
// folded with a butterfly, the four waves are added in wave order, and the split-K partial sums go
// to part[ks][row][h*r + j], the layout the scan and the finalisation read.
template <typename T, int NBR>
__global__ __launch_bounds__(256) void project_columns(const T *__restrict__ W, const T *__restrict__ x,
                                                       const int32_t *__restrict__ idx,
                                                       float *__restrict__ part, int B, int D, int d,
                                                       int r, int LPR, int LPRp, int k_per, int Bpad,
                                                       int Cpad) {
  constexpr int TPL = Elem<T>::TPL;
  constexpr int KC = 512;                  // K rows staged per chunk
  constexpr int U = NBR <= 8 ? 8 : 4;      // loads in flight per lane
  typedef typename Elem<T>::vec vec;
  __shared__ float xs[NBR * KC];
  __shared__ float red[NBR * 512];
  const int h = blockIdx.x, ks = blockIdx.y, n0 = blockIdx.z * NBR;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int RPW = 64 / LPRp;
  const int sub = lane / LPRp, li = lane % LPRp;
  const bool active = li < LPR;
  const int k0 = ks * k_per, k1 = min(D, k0 + k_per);
  float acc[NBR][TPL];
#pragma unroll
  for (int b = 0; b < NBR; ++b)
#pragma unroll
    for (int e = 0; e < TPL; ++e) acc[b][e] = 0.f;
  const T *wcol = W + (long)h * d + (active ? li : 0) * TPL;
  for (int kc = k0; kc < k1; kc += KC) {
    const int kn = min(KC, k1 - kc);
    __syncthreads();
    for (int b = 0; b < NBR; ++b) {
      const int row = n0 + b;
      for (int kk = tid; kk < kn; kk += 256)
        xs[b * KC + kk] = row < B ? (float)x[(long)row * D + kc + kk] : 0.f;
    }
    __syncthreads();
    const int steps = (kn + 4 * RPW - 1) / (4 * RPW);
    for (int s0 = 0; s0 < steps; s0 += U) {
      vec v[U];
      int kk[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int k = ((s0 + u) * 4 + w) * RPW + sub;
        const bool ok = active && k < kn;
        kk[u] = min(k, kn - 1);
        vec z = {};
        v[u] = ok ? *reinterpret_cast<const vec *>(wcol + (long)(kc + kk[u]) * D) : z;
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float wf[TPL];
#pragma unroll
        for (int e = 0; e < TPL; ++e) wf[e] = (float)v[u][e];
#pragma unroll
        for (int b = 0; b < NBR; ++b) {
          const float xv = xs[b * KC + kk[u]];
#pragma unroll
          for (int e = 0; e < TPL; ++e) acc[b][e] = fmaf(xv, wf[e], acc[b][e]);
        }
      }
    }
  }
  // rows of one wave
  for (int o = LPRp; o < 64; o <<= 1) {
#pragma unroll
    for (int b = 0; b < NBR; ++b)
#pragma unroll
      for (int e = 0; e < TPL; ++e) acc[b][e] += __shfl_xor(acc[b][e], o, 64);
  }
  // the four waves, in wave order
  for (int ww = 0; ww < 4; ++ww) {
    if (w == ww && sub == 0 && active) {
#pragma unroll
      for (int b = 0; b < NBR; ++b)
#pragma unroll
        for (int e = 0; e < TPL; ++e) {
          const int at = b * 512 + li * TPL + e;
          red[at] = (ww == 0 ? 0.f : red[at]) + acc[b][e];
        }
    }
    __syncthreads();
  }
  for (int i = tid; i < NBR * r; i += 256) {
    const int b = i / r, j = i % r;
    const int row = n0 + b;
    const int col = min(max(idx[h * r + j], 0), d - 1);
    if (row < Bpad) part[((long)ks * Bpad + row) * Cpad + h * r + j] = red[b * 512 + col];
  }
}

// The same for half precision on the matrix cores (D a multiple of 128): workgroup (128-column
// block, ks, batch blocks).  Lane (n = lane%16, kg = lane/16) of a wave loads, for 8 consecutive
// rows k, the 16 bytes holding columns 8n .. 8n+7 of the block (16 lanes cover one 256-byte row
// piece, a wave-wide step covers 32 rows), turns its 8x8 block of halves around in registers so
// that each of its 8 columns has 8 consecutive k, and issues 8 MFMAs 16x16x32 per batch block:
// MFMA j multiplies columns {8m + j} (A operand, m = lane%16) with the x fragment (B operand, 16
// batch rows).  Result register v of lane l in MFMA j: column 8*(4*(l/16) + v) + j, batch row l%16.
// The four waves take every fourth step; their sums are added in wave order through LDS.
template <int NB>
__global__ __launch_bounds__(256) void project_columns_mfma(const half_t *__restrict__ W,
                                                            const half_t *__restrict__ x,
                                                            const int32_t *__restrict__ idx,
                                                            float *__restrict__ part, int B, int D,
                                                            int H, int d, int r, int k_per, int Bpad,
                                                            int Cpad) {
  constexpr int RS = 129;                   // row stride of the LDS result tile (floats)
  __shared__ float red[NB * 16 * RS];
  const int cb = blockIdx.x, ks = blockIdx.y, nb0 = blockIdx.z * NB;
  const int tid = threadIdx.x, w = tid >> 6, lane = tid & 63;
  const int n = lane & 15, kg = lane >> 4;
  const int k0 = ks * k_per, k1 = min(D, k0 + k_per);      // both multiples of 32
  floatx4 acc[NB][8];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
  const half8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
  const half_t *wp = W + (long)cb * 128 + n * 8;
  // two steps per pass: 16 row loads of a lane are in flight before the first MFMA
  for (int kb = k0 + w * 32; kb < k1; kb += 256) {
    half8 rows[2][8], xf[2][NB];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int kt = kb + t * 128 + kg * 8;
      const bool ok = kt < k1;
#pragma unroll
      for (int e = 0; e < 8; ++e) rows[t][e] = ok ? *reinterpret_cast<const half8 *>(wp + (long)(kt + e) * D) : zero;
#pragma unroll
      for (int i = 0; i < NB; ++i) {
        const int row = (nb0 + i) * 16 + n;
        xf[t][i] = (ok && row < B) ? *reinterpret_cast<const half8 *>(x + (long)row * D + kt) : zero;
      }
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      if (kb + t * 128 < k1) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          half8 a;
#pragma unroll
          for (int e = 0; e < 8; ++e) a[e] = rows[t][e][j];
#pragma unroll
          for (int i = 0; i < NB; ++i)
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, xf[t][i], acc[i][j], 0, 0, 0);
        }
      }
    }
  }
  for (int ww = 0; ww < 4; ++ww) {
    if (w == ww) {
#pragma unroll
      for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int at = (i * 16 + n) * RS + 8 * (4 * kg + v) + j;
            red[at] = (ww == 0 ? 0.f : red[at]) + acc[i][j][v];
          }
    }
    __syncthreads();
  }
  // kept columns that fall into this block, for the heads that overlap it
  const int c_lo = cb * 128;
  const int h_lo = c_lo / d, h_hi = min(H - 1, (c_lo + 127) / d);
  for (int i = h_lo * r + tid; i < (h_hi + 1) * r; i += 256) {
    const int col = (i / r) * d + min(max(idx[i], 0), d - 1) - c_lo;
    if (col < 0 || col >= 128) continue;
    for (int b = 0; b < NB * 16; ++b) {
      const int row = nb0 * 16 + b;
      if (row < Bpad) part[((long)ks * Bpad + row) * Cpad + i] = red[b * RS + col];
    }
  }
}

// ---- finalisation -------------------------------------------------------------------------------
// folded: q_p[b,h,j] = bias[h*r+j] + sum_s part[s][b][h*r+j]
// rope:   q[c] = bias[h*d+c] + sum_s part[s][b][h*d+c]; rotate pairs (c, c+d/2) by
//         pos[b]*theta^(-2c/d) (angle in double: positions reach 1e5 where float loses the phase);
//         q_p[b,h,k] = sum_c q_rot[c] * A_p[h][c][k]
// (Section 4.3 "Decoding Stage" for models whose skew cannot be folded into W_Q.)
__global__ __launch_bounds__(256) void finalize_query(const float *__restrict__ part,
                                                      const float *__restrict__ bias,
                                                      const float *__restrict__ A_p,
                                                      const int32_t *__restrict__ pos,
                                                      float *__restrict__ q_p, int H, int d, int r,
                                                      int KS, long ks_stride, int Cpad, int rope,
                                                      double freq_step /* -(2/d) log2(theta) */) {
  __shared__ float q[512];
  __shared__ float qr[512];
  __shared__ float psum[256];
  const int bh = blockIdx.x, b = bh / H, h = bh % H;
  const int t = threadIdx.x;
  if (!rope) {
    // split-K partial sums: all loads of a column issued together, added in a fixed order
    for (int c = t; c < r; c += 256) {
      const float *p = part + (long)b * Cpad + (long)h * r + c;
      float v[IG_KS_MAX];
#pragma unroll
      for (int s = 0; s < IG_KS_MAX; ++s) v[s] = (s < KS) ? p[s * ks_stride] : 0.f;
      float acc = bias ? bias[h * r + c] : 0.f;
#pragma unroll
      for (int s = 0; s < IG_KS_MAX; ++s) acc += v[s];
      q_p[(long)bh * r + c] = acc;
    }
    return;
  }
  // Rotary model.  The block is one chain of dependent steps, so everything it reads is put in
  // flight before the first step: the partial sums of its (up to two) columns, the position, and
  // the thread's rows of A_p, which do not depend on the query at all.
  float v[2][IG_KS_MAX], bs[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int c = t + 256 * u;
#pragma unroll
    for (int s = 0; s < IG_KS_MAX; ++s) v[u][s] = 0.f;
    bs[u] = 0.f;
    if (c < d) {
      const float *p = part + (long)b * Cpad + (long)h * d + c;
#pragma unroll
      for (int s = 0; s < IG_KS_MAX; ++s)
        if (s < KS) v[u][s] = p[s * ks_stride];
      if (bias) bs[u] = bias[h * d + c];
    }
  }
  const int position = pos[b];
  // q_p[k] = sum_c qr[c] * A_p[h][c][k]: the threads are G groups of r; group g sums its share of
  // the rows c for output k (reads of A_p coalesce over k), then the groups are added in order
  const int G = 256 / r;                      // r <= 256
  const int k = t % r, g = t / r;
  const int per = (d + G - 1) / G;
  const int c0 = g < G ? min(d, g * per) : d, c1 = g < G ? min(d, (g + 1) * per) : d;
  constexpr int PF = 24;
  const float *ap = A_p + (long)h * d * r + k;
  float apf[PF];
#pragma unroll
  for (int i = 0; i < PF; ++i) {
    apf[i] = 0.f;
    if (c0 + i < c1) apf[i] = ap[(long)(c0 + i) * r];
  }
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int c = t + 256 * u;
    float acc = bs[u];
#pragma unroll
    for (int s = 0; s < IG_KS_MAX; ++s) acc += v[u][s];
    if (c < d) q[c] = acc;
  }
  __syncthreads();
  const int half = d / 2;
  for (int c = t; c < half; c += 256) {
    double sn, cs;
    rope_sincos((double)position * exp2((double)c * freq_step), &sn, &cs);
    float a = q[c], bb = q[c + half];
    qr[c] = (float)((double)a * cs - (double)bb * sn);
    qr[c + half] = (float)((double)bb * cs + (double)a * sn);
  }
  __syncthreads();
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < PF; ++i)
    if (c0 + i < c1) acc = fmaf(qr[c0 + i], apf[i], acc);
  for (int c = c0 + PF; c < c1; ++c) acc = fmaf(qr[c], ap[(long)c * r], acc);
  psum[t] = acc;
  __syncthreads();
  if (t < r) {
    float tot = 0.f;
    for (int gg = 0; gg < G; ++gg) tot += psum[gg * r + t];
    q_p[(long)bh * r + t] = tot;
  }
}

}  // namespace

int ig_launch_wq_build(ig_ctx *ctx, const ig_desc *d, const ProjGeom &g, const void *Wq,
                       const int32_t *idx, void *wq, hipStream_t s) {
  const int D = d->H * d->d;
  const int32_t *ix = d->rope ? nullptr : idx;
  if (g.mfma) {
    long total = (long)g.nCblk * g.nKblk * 64;
    auto k = wq_build_mfma;
    IG_LAUNCH(ctx, IG_K_BUILD, k, dim3((unsigned)((total + 255) / 256)), dim3(256), s,
              (const half_t *)Wq, ix, (half8 *)wq, D, (int)d->d, (int)d->r, g.C, g.nCblk, g.nKblk);
  } else if (d->dtype == IG_F16) {
    long total = (long)D * g.Cpad;
    auto k = wq_build_plain<half_t>;
    IG_LAUNCH(ctx, IG_K_BUILD, k, dim3((unsigned)((total + 255) / 256)), dim3(256), s,
              (const half_t *)Wq, ix, (half_t *)wq, D, (int)d->d, (int)d->r, g.C, g.Cpad);
  } else {
    long total = (long)D * g.Cpad;
    auto k = wq_build_plain<float>;
    IG_LAUNCH(ctx, IG_K_BUILD, k, dim3((unsigned)((total + 255) / 256)), dim3(256), s,
              (const float *)Wq, ix, (float *)wq, D, (int)d->d, (int)d->r, g.C, g.Cpad);
  }
  return IG_OK;
}

int ig_launch_project(ig_ctx *ctx, const ig_desc *d, const ProjGeom &g, const void *x,
                      const void *wq, float *part, hipStream_t s) {
  const int D = d->H * d->d;
  if (g.mfma) {
    long waves = (long)g.nCblk * g.KS;
    dim3 block(256);
    if (g.NBtot == 1) {
      auto k = project_mfma<1>;
      IG_LAUNCH(ctx, IG_K_PROJECT, k, dim3((unsigned)((waves + 3) / 4), 1), block, s,
                (const half8 *)wq, (const half_t *)x, part, (int)d->B, D, g.nCblk, g.nKblk, g.kb_per,
                g.KS, g.Bpad, g.Cpad);
    } else if (g.NBtot == 2 && g.kb_per <= 16) {
      // 17..32 batch rows: x fragments through LDS, a wave's whole K slice of weights in flight
      auto k = project_mfma_shared<2, 16>;
      const size_t lds = (size_t)32 * (g.kb_per * 4 + 1) * 16;
      const dim3 grid((unsigned)((g.nCblk + 3) / 4), (unsigned)g.KS);
      IG_LAUNCH_LDS(ctx, IG_K_PROJECT, k, grid, block, lds, s, (const half8 *)wq, (const half_t *)x, part,
                    (int)d->B, D, g.nCblk, g.nKblk, g.kb_per, g.Bpad, g.Cpad);
    } else if (g.NBtot == 2) {
      auto k = project_mfma<2>;
      IG_LAUNCH(ctx, IG_K_PROJECT, k, dim3((unsigned)((waves + 3) / 4), 1), block, s,
                (const half8 *)wq, (const half_t *)x, part, (int)d->B, D, g.nCblk, g.nKblk, g.kb_per,
                g.KS, g.Bpad, g.Cpad);
    } else {
      auto k = project_mfma<4>;
      IG_LAUNCH(ctx, IG_K_PROJECT, k, dim3((unsigned)((waves + 3) / 4), (unsigned)((g.NBtot + 3) / 4)),
                block, s, (const half8 *)wq, (const half_t *)x, part, (int)d->B, D, g.nCblk, g.nKblk,
                g.kb_per, g.KS, g.Bpad, g.Cpad);
    }
  } else {
    dim3 grid((g.Cpad + 63) / 64, g.KS, g.NBtot), block(64);
    if (d->dtype == IG_F16) {
      auto k = project_fma<half_t>;
      IG_LAUNCH(ctx, IG_K_PROJECT, k, grid, block, s, (const half_t *)wq, (const half_t *)x, part,
                (int)d->B, D, g.kb_per, g.Bpad, g.Cpad);
    } else {
      auto k = project_fma<float>;
      IG_LAUNCH(ctx, IG_K_PROJECT, k, grid, block, s, (const float *)wq, (const float *)x, part,
                (int)d->B, D, g.kb_per, g.Bpad, g.Cpad);
    }
  }
  return IG_OK;
}

// Split of the index-only projection: enough workgroups for two per compute unit.  Half precision
// with D a multiple of 128 runs on the matrix cores (column blocks of 128, K slices that are
// multiples of 32, up to 4 batch blocks of 16 per workgroup); everything else on the FMA kernel
// (one head per workgroup, 8 or 16 batch rows).
static bool proj_columns_mfma(const ig_desc *d) { return d->dtype == IG_F16 && (d->H * d->d) % 128 == 0; }

int ig_proj_columns_ks(const ig_desc *d, int *k_per) {
  const int D = d->H * d->d;
  int wgs, unit;
  if (proj_columns_mfma(d)) {
    const int nbtot = (d->B + 15) / 16;
    wgs = (D / 128) * ((nbtot + 3) / 4);
    unit = 32;
  } else {
    const int nbr = d->B <= 8 ? 8 : 16;
    wgs = d->H * ((d->B + nbr - 1) / nbr);
    unit = 1;
  }
  const int units = D / unit;
  int ks = (512 + wgs - 1) / wgs;
  if (ks > IG_KS_MAX) ks = IG_KS_MAX;
  if (ks > units) ks = units;
  if (ks < 1) ks = 1;
  *k_per = (units + ks - 1) / ks * unit;
  return (D + *k_per - 1) / *k_per;
}

int ig_launch_project_columns(ig_ctx *ctx, const ig_desc *d, const ProjGeom &g, const void *x,
                              const void *W, const int32_t *idx, float *part, hipStream_t s) {
  const int D = d->H * d->d;
  int k_per = 0;
  const int KS = ig_proj_columns_ks(d, &k_per);
  if (proj_columns_mfma(d)) {
    const int nbtot = (d->B + 15) / 16;
    const int nb = nbtot == 1 ? 1 : (nbtot == 2 ? 2 : 4);
    dim3 grid(D / 128, KS, (nbtot + nb - 1) / nb), block(256);
#define PM_CASE(NB)                                                                                \
  {                                                                                                \
    auto k = project_columns_mfma<NB>;                                                             \
    IG_LAUNCH(ctx, IG_K_PROJECT, k, grid, block, s, (const half_t *)W, (const half_t *)x, idx,     \
              part, (int)d->B, D, (int)d->H, (int)d->d, (int)d->r, k_per, g.Bpad, g.Cpad);         \
    return IG_OK;                                                                                  \
  }
    if (nb == 1) PM_CASE(1)
    if (nb == 2) PM_CASE(2)
    PM_CASE(4)
#undef PM_CASE
  }
  const int row_bytes = d->d * ig_elem_bytes(d->dtype);
  if (row_bytes % 16 || row_bytes / 16 > 64 || d->d > 512)
    return ig_fail(ctx, IG_ESHAPE, "index-only projection: d = %d needs 16-byte rows of at most 1 KiB", d->d);
  const int LPR = row_bytes / 16;
  int LPRp = 1;
  while (LPRp < LPR) LPRp <<= 1;
  const int nbr = d->B <= 8 ? 8 : 16;
  dim3 grid(d->H, KS, (d->B + nbr - 1) / nbr), block(256);
#define PC_CASE(T, NBR)                                                                            \
  {                                                                                                \
    auto k = project_columns<T, NBR>;                                                              \
    IG_LAUNCH(ctx, IG_K_PROJECT, k, grid, block, s, (const T *)W, (const T *)x, idx, part,         \
              (int)d->B, D, (int)d->d, (int)d->r, LPR, LPRp, k_per, g.Bpad, g.Cpad);               \
    return IG_OK;                                                                                  \
  }
  if (d->dtype == IG_F16) {
    if (nbr == 8) PC_CASE(half_t, 8)
    PC_CASE(half_t, 16)
  }
  if (nbr == 8) PC_CASE(float, 8)
  PC_CASE(float, 16)
#undef PC_CASE
}

int ig_launch_finalize(ig_ctx *ctx, const ig_desc *d, const ProjGeom &g, const float *part,
                       const float *bias, const float *A_p, const int32_t *pos, float *q_p,
                       hipStream_t s) {
  if (d->rope && d->d > 512) return ig_fail(ctx, IG_ESHAPE, "rope: d = %d exceeds 512", d->d);
  auto k = finalize_query;
  IG_LAUNCH(ctx, IG_K_FINALIZE, k, dim3(d->B * d->H), dim3(256), s, part, bias, A_p, pos, q_p,
            (int)d->H, (int)d->d, (int)d->r, g.KS, (long)g.Bpad * g.Cpad, g.Cpad, (int)d->rope,
            d->rope ? -2.0 / (double)d->d * log2((double)d->rope_theta) : 0.0);
  return IG_OK;
}
