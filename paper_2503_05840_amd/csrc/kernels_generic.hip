// Generic vector-ALU kernels of the slim-attention decode step (gfx950).
//
// These handle every supported shape in fp32 arithmetic for both cache element types
// (fp32, bf16) and are the path for fp32 caches; the bf16 fast kernels live in
// kernels_bf16.hip.  Steps, in the paper's terms:
//   head_scores   : softmax arguments q_i K_i^T / sqrt(d_k)                 (eq. 2)
//   weighted_sum  : [softmax(.) K], the full-width weighted sum of K rows   (eq. 7, option 2)
//                   per split of the context, with a local max (flash-decoding style)
//   combine       : log-sum-exp merge of the splits and the 1/l normalisation
//   project       : ... W_KV,i per head                                     (eq. 7, option 2)
//   vanilla_*     : softmax(.) V_i reading both caches                      (eq. 2; Table 2 "Vanilla")
//   dense_scores  : (q_i W_K,i^T) X^T for the X-cache scheme                (non-square section, Fig. 4)
#include "slim_kernels.h"
#include "device_common.h"

#include <type_traits>

#include <math.h>

namespace slim {
namespace {

struct F32 {
  using elem = float;
  static constexpr int VEC = 4;
  static __device__ __forceinline__ void load(const elem* p, float (&v)[4]) {
    const float4 x = *reinterpret_cast<const float4*>(p);
    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
  }
  // the same for data that is read once (non-temporal: does not displace what is reused)
  static __device__ __forceinline__ void load_stream(const elem* p, float (&v)[4]) {
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4 x = __builtin_nontemporal_load(reinterpret_cast<const f4*>(p));
    v[0] = x[0]; v[1] = x[1]; v[2] = x[2]; v[3] = x[3];
  }
  static __device__ __forceinline__ float one(const elem* p) { return *p; }
  static __device__ __forceinline__ void two(const elem* p, float& a, float& b) {
    const float2 x = *reinterpret_cast<const float2*>(p);
    a = x.x; b = x.y;
  }
  static __device__ __forceinline__ void store_two(elem* p, float a, float b) {
    *reinterpret_cast<float2*>(p) = make_float2(a, b);
  }
};

struct BF16 {
  using elem = uint16_t;
  static constexpr int VEC = 8;
  static __device__ __forceinline__ void load(const elem* p, float (&v)[8]) {
    const uint4 x = *reinterpret_cast<const uint4*>(p);
    v[0] = __uint_as_float(x.x << 16); v[1] = __uint_as_float(x.x & 0xffff0000u);
    v[2] = __uint_as_float(x.y << 16); v[3] = __uint_as_float(x.y & 0xffff0000u);
    v[4] = __uint_as_float(x.z << 16); v[5] = __uint_as_float(x.z & 0xffff0000u);
    v[6] = __uint_as_float(x.w << 16); v[7] = __uint_as_float(x.w & 0xffff0000u);
  }
  static __device__ __forceinline__ void load_stream(const elem* p, float (&v)[8]) {
    typedef unsigned u4 __attribute__((ext_vector_type(4)));
    const u4 x = __builtin_nontemporal_load(reinterpret_cast<const u4*>(p));
    v[0] = __uint_as_float(x[0] << 16); v[1] = __uint_as_float(x[0] & 0xffff0000u);
    v[2] = __uint_as_float(x[1] << 16); v[3] = __uint_as_float(x[1] & 0xffff0000u);
    v[4] = __uint_as_float(x[2] << 16); v[5] = __uint_as_float(x[2] & 0xffff0000u);
    v[6] = __uint_as_float(x[3] << 16); v[7] = __uint_as_float(x[3] & 0xffff0000u);
  }
  static __device__ __forceinline__ float one(const elem* p) {
    return __uint_as_float(((uint32_t)*p) << 16);
  }
  static __device__ __forceinline__ void two(const elem* p, float& a, float& b) {
    const uint32_t x = *reinterpret_cast<const uint32_t*>(p);
    a = __uint_as_float(x << 16); b = __uint_as_float(x & 0xffff0000u);
  }
  static __device__ __forceinline__ void store_two(elem* p, float a, float b) {   // round to nearest even
    const uint32_t lo = __builtin_bit_cast(uint16_t, (__bf16)a), hi = __builtin_bit_cast(uint16_t, (__bf16)b);
    *reinterpret_cast<uint32_t*>(p) = lo | (hi << 16);
  }
};


// ------------------------------------------------------------------------------------------------
// head_scores: one wave per row; lanes stride over the row in 16-byte vectors, partial dot
// products go to LDS and are summed per head (works for any d_k that is a multiple of VEC).
// ------------------------------------------------------------------------------------------------
constexpr int HS_ROWS = 32;   // rows per workgroup (4 waves x 8 rows)

template <class ET>
__global__ __launch_bounds__(256) void head_scores_kernel(
    const float* __restrict__ q, long q_bstride, const typename ET::elem* __restrict__ M,
    long m_bstride, long row_pitch, const int32_t* __restrict__ rows_per_b, int rows, int e, int H,
    int d_k, float scale, float* __restrict__ S, long s_bstride, const float* __restrict__ rope) {
  extern __shared__ float smem[];
  constexpr int VEC = ET::VEC;
  const int nvec = e / VEC;
  float* q_s = smem;                 // [e]
  float* part = smem + e;            // [4][nvec]
  const int b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nrows = seq_len_of(rows_per_b, b, rows);
  const int r0 = blockIdx.x * HS_ROWS;
  if (r0 >= nrows) return;
  for (int i = tid; i < e; i += 256) q_s[i] = q[b * q_bstride + i];
  __syncthreads();
  const int cpk = d_k / VEC;
  float* mypart = part + wave * nvec;
  for (int it = 0; it < HS_ROWS / 4; ++it) {
    const int r = r0 + it * 4 + wave;
    const bool valid = r < nrows;
    if (valid) {
      const typename ET::elem* row = M + b * m_bstride + (long)r * row_pitch;
      for (int ci = lane; ci < nvec; ci += 64) {
        float v[VEC];
        ET::load(row + ci * VEC, v);
        float acc = 0.f;
        if (rope) {
          // RoPE appendix, option 1: the raw row is rotated by its position r for the score only.
          // With (y1, y2) = (x1 c + x2 s, -x1 s + x2 c):  q1 y1 + q2 y2 = c (q1 x1 + q2 x2) + s (q1 x2 - q2 x1).
          const float* cs = rope + ((size_t)r * (d_k / 2) + (ci * VEC) % d_k / 2) * 2;
#pragma unroll
          for (int j = 0; j < VEC; j += 2) {
            const float q1 = q_s[ci * VEC + j], q2 = q_s[ci * VEC + j + 1];
            acc = fmaf(cs[j], fmaf(q1, v[j], q2 * v[j + 1]), acc);
            acc = fmaf(cs[j + 1], fmaf(q1, v[j + 1], -q2 * v[j]), acc);
          }
        } else {
#pragma unroll
          for (int j = 0; j < VEC; ++j) acc = fmaf(v[j], q_s[ci * VEC + j], acc);
        }
        mypart[ci] = acc;
      }
    }
    __syncthreads();
    if (valid) {
      for (int h = lane; h < H; h += 64) {
        float s = 0.f;
        for (int j = 0; j < cpk; ++j) s += mypart[h * cpk + j];
        S[b * s_bstride + (long)h * rows + r] = s * scale;
      }
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------------
// dense_scores: S[b][h][t] = scale * sum_c qt[b][h][c] X[b][t][c]; LDS-tiled 64 t x 32 h x 64 c.
// ------------------------------------------------------------------------------------------------
constexpr int DS_T = 64, DS_H = 32, DS_C = 64;

template <class ET>
__global__ __launch_bounds__(256) void dense_scores_kernel(
    const float* __restrict__ qt, const typename ET::elem* __restrict__ X, long x_bstride,
    int d_model, const int32_t* __restrict__ seq_lens, int T, int H, float scale,
    float* __restrict__ S) {
  __shared__ float Xs[DS_T][DS_C + 1];
  __shared__ float Qs[DS_H][DS_C + 1];
  constexpr int VEC = ET::VEC;
  const int b = blockIdx.z;
  const int len = seq_len_of(seq_lens, b, T);
  const int t0 = blockIdx.x * DS_T, h0 = blockIdx.y * DS_H;
  if (t0 >= len) return;
  const int tid = threadIdx.x;
  const int tt = tid & 63, hq = tid >> 6;      // 8 heads per thread
  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;
  for (int c0 = 0; c0 < d_model; c0 += DS_C) {
    // X tile: DS_T rows x DS_C cols in vectors
    constexpr int VPR = DS_C / VEC;            // vectors per row
    for (int i = tid; i < DS_T * VPR; i += 256) {
      const int r = i / VPR, cv = (i % VPR) * VEC;
      float v[VEC];
#pragma unroll
      for (int j = 0; j < VEC; ++j) v[j] = 0.f;
      const int t = t0 + r;
      if (t < len && c0 + cv < d_model) ET::load(X + b * x_bstride + (long)t * d_model + c0 + cv, v);
#pragma unroll
      for (int j = 0; j < VEC; ++j) Xs[r][cv + j] = v[j];
    }
    for (int i = tid; i < DS_H * DS_C; i += 256) {
      const int hh = i / DS_C, cc = i % DS_C;
      const int h = h0 + hh, c = c0 + cc;
      Qs[hh][cc] = (h < H && c < d_model) ? qt[((long)b * H + h) * d_model + c] : 0.f;
    }
    __syncthreads();
#pragma unroll 8
    for (int cc = 0; cc < DS_C; ++cc) {
      const float x = Xs[tt][cc];
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] = fmaf(x, Qs[hq * 8 + j][cc], acc[j]);
    }
    __syncthreads();
  }
  const int t = t0 + tt;
  if (t < len) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int h = h0 + hq * 8 + j;
      if (h < H) S[((long)b * H + h) * T + t] = acc[j] * scale;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// weighted_sum: grid (colblocks * headblocks, nsplit, B).  Each workgroup owns 512 columns
// (2 per thread) and up to 32 heads, walks its split of the context in tiles of 32 rows:
// P = exp(S - m_local) into LDS, then acc[h][c] += P[t][h] * M[t][c].
// ------------------------------------------------------------------------------------------------
constexpr int WS_HB = 32, WS_TT = 32, WS_COLS = 512;

__host__ __device__ inline int split_rows(int T, int nsplit) {
  int ts = (T + nsplit - 1) / nsplit;
  return (ts + 31) & ~31;
}

template <class ET>
__global__ __launch_bounds__(256) void weighted_sum_kernel(
    const float* __restrict__ S, const typename ET::elem* __restrict__ M, long m_bstride, int width,
    const int32_t* __restrict__ seq_lens, int T, int H, int nsplit, int ncolblk,
    float* __restrict__ Cpart, float* __restrict__ mpart, float* __restrict__ lpart) {
  __shared__ __attribute__((aligned(16))) float P[WS_TT][WS_HB];
  __shared__ float m_s[WS_HB];
  const int b = blockIdx.z, sp = blockIdx.y;
  const int cb = blockIdx.x % ncolblk, hb = blockIdx.x / ncolblk;
  const int tid = threadIdx.x;
  const int len = seq_len_of(seq_lens, b, T);
  const int ts = split_rows(T, nsplit);
  const int t0 = sp * ts;
  const int t1 = min(len, t0 + ts);
  const int h0 = hb * WS_HB;
  const int c = cb * WS_COLS + tid * 2;
  const bool col_ok = c < width;               // width is even (multiple of VEC)

  // phase 0: local max per head
  const int hh = tid >> 3, sub = tid & 7;
  const int h = h0 + hh;
  const float* Srow = S + ((long)b * H + (h < H ? h : 0)) * T;
  float mx = NEG_INF;
  if (h < H)
    for (int t = t0 + sub; t < t1; t += 8) mx = fmaxf(mx, Srow[t]);
  mx = fmaxf(mx, __shfl_xor(mx, 1));
  mx = fmaxf(mx, __shfl_xor(mx, 2));
  mx = fmaxf(mx, __shfl_xor(mx, 4));
  if (sub == 0) m_s[hh] = mx;
  __syncthreads();

  float acc[WS_HB][2];
#pragma unroll
  for (int i = 0; i < WS_HB; ++i) acc[i][0] = acc[i][1] = 0.f;
  float lsum = 0.f;
  const typename ET::elem* Mb = M + b * m_bstride;

  for (int tb = t0; tb < t1; tb += WS_TT) {
#pragma unroll
    for (int i = 0; i < WS_TT / 8; ++i) {
      const int tt = sub + i * 8;
      const int t = tb + tt;
      float p = 0.f;
      if (h < H && t < t1) p = __expf(Srow[t] - mx);
      P[tt][hh] = p;
      lsum += p;
    }
    __syncthreads();
    const int nt = min(WS_TT, t1 - tb);
    if (col_ok) {
      for (int tt = 0; tt < nt; ++tt) {
        float k0, k1;
        ET::two(Mb + (long)(tb + tt) * width + c, k0, k1);
#pragma unroll
        for (int g = 0; g < WS_HB; g += 4) {
          const float4 pv = *reinterpret_cast<const float4*>(&P[tt][g]);
          acc[g + 0][0] = fmaf(pv.x, k0, acc[g + 0][0]); acc[g + 0][1] = fmaf(pv.x, k1, acc[g + 0][1]);
          acc[g + 1][0] = fmaf(pv.y, k0, acc[g + 1][0]); acc[g + 1][1] = fmaf(pv.y, k1, acc[g + 1][1]);
          acc[g + 2][0] = fmaf(pv.z, k0, acc[g + 2][0]); acc[g + 2][1] = fmaf(pv.z, k1, acc[g + 2][1]);
          acc[g + 3][0] = fmaf(pv.w, k0, acc[g + 3][0]); acc[g + 3][1] = fmaf(pv.w, k1, acc[g + 3][1]);
        }
      }
    }
    __syncthreads();
  }
  lsum += __shfl_xor(lsum, 1);
  lsum += __shfl_xor(lsum, 2);
  lsum += __shfl_xor(lsum, 4);
  const long pbase = ((long)b * nsplit + sp) * H;
  if (cb == 0 && sub == 0 && h < H) {
    mpart[pbase + h] = mx;
    lpart[pbase + h] = lsum;
  }
  if (col_ok) {
#pragma unroll
    for (int i = 0; i < WS_HB; ++i) {
      const int hi = h0 + i;
      if (hi < H)
        *reinterpret_cast<float2*>(Cpart + (pbase + hi) * width + c) = make_float2(acc[i][0], acc[i][1]);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// combine: merge the splits (log-sum-exp weights) and normalise.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void combine_kernel(const float* __restrict__ Cpart,
                                                      const float* __restrict__ mpart,
                                                      const float* __restrict__ lpart, int nsplit,
                                                      int H, int width, float* __restrict__ Cn) {
  const int b = blockIdx.y;
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= (long)H * width) return;
  const int h = (int)(i / width);
  const int c = (int)(i % width);
  float m = NEG_INF;
  for (int s = 0; s < nsplit; ++s) m = fmaxf(m, mpart[((long)b * nsplit + s) * H + h]);
  float num = 0.f, den = 0.f;
  for (int s = 0; s < nsplit; ++s) {
    const long pb = ((long)b * nsplit + s) * H + h;
    const float ms = mpart[pb];
    const float w = (ms == NEG_INF) ? 0.f : __expf(ms - m);
    num = fmaf(w, Cpart[pb * width + c], num);
    den = fmaf(w, lpart[pb], den);
  }
  Cn[((long)b * H + h) * width + c] = num / den;
}

// ------------------------------------------------------------------------------------------------
// project: out[b][n] = sum_c Cn[b][n/d_k][c] W[c][n].  Workgroup = 64 output columns x 4 batch
// rows; its 16 waves interleave over c, eight rows of W in flight per wave, and are summed through
// LDS in a fixed order.
// ------------------------------------------------------------------------------------------------
constexpr int PROJ_WAVES = 16, PROJ_UNROLL = 8;

template <class ET>
__global__ __launch_bounds__(PROJ_WAVES * 64) void project_kernel(const float* __restrict__ Cn,
                                                                 const typename ET::elem* __restrict__ W,
                                                                 int rows, int e, int H, int d_k,
                                                                 float* __restrict__ out, int B) {
  __shared__ float red[PROJ_WAVES][4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = blockIdx.x * 64 + lane;
  const int b0 = blockIdx.y * 4;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  if (n < e) {
    const int h = n / d_k;
    const float* cp[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) cp[j] = Cn + ((long)min(b0 + j, B - 1) * H + h) * rows;
    const typename ET::elem* wn = W + n;
    int c = wave;
    const bool one_row = b0 + 1 >= B;                  // (a single sequence: no loads for the three rows that repeat it)
    for (; c + (PROJ_UNROLL - 1) * PROJ_WAVES < rows; c += PROJ_UNROLL * PROJ_WAVES) {
      float w[PROJ_UNROLL];
#pragma unroll
      for (int u = 0; u < PROJ_UNROLL; ++u) w[u] = ET::one(wn + (long)(c + u * PROJ_WAVES) * e);
      if (one_row) {
#pragma unroll
        for (int u = 0; u < PROJ_UNROLL; ++u) acc[0] = fmaf(cp[0][c + u * PROJ_WAVES], w[u], acc[0]);
      } else {
#pragma unroll
        for (int u = 0; u < PROJ_UNROLL; ++u)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[j] = fmaf(cp[j][c + u * PROJ_WAVES], w[u], acc[j]);
      }
    }
    for (; c < rows; c += PROJ_WAVES) {
      const float w = ET::one(wn + (long)c * e);
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = fmaf(cp[j][c], w, acc[j]);
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) red[wave][j][lane] = acc[j];
  __syncthreads();
  if (wave == 0 && n < e) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (b0 + j >= B) continue;
      float sum = 0.f;
#pragma unroll
      for (int ww = 0; ww < PROJ_WAVES; ++ww) sum += red[ww][j][lane];
      out[(long)(b0 + j) * e + n] = sum;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// append: the new token's projected key (and value) row of every sequence goes into the cache at
// row len_b - 1 (the generate-phase description under Fig. 2).  One thread per adjacent column pair.
// With a rotary table the token sits at position len_b - 1: its query is rotated there in place,
// and its key too when the cache stores rotated keys (vanilla); a slim cache keeps the raw key.
// ------------------------------------------------------------------------------------------------
template <class ET>
__global__ __launch_bounds__(256) void append_kernel(
    const float* __restrict__ knew, const float* __restrict__ vnew, typename ET::elem* __restrict__ K,
    typename ET::elem* __restrict__ V, long bstride, const int32_t* __restrict__ seq_lens, int T, int d,
    int d_k, const float* __restrict__ rope, float* __restrict__ q, int rotate_k) {
  const int b = blockIdx.y;
  const int col = (blockIdx.x * 256 + threadIdx.x) * 2;
  const int len = seq_len_of(seq_lens, b, T);
  if (col >= d || len < 1) return;
  const int pos = len - 1;
  float k1 = knew[(long)b * d + col], k2 = knew[(long)b * d + col + 1];
  if (rope) {
    const float* cs = rope + ((size_t)pos * (d_k / 2) + (col % d_k) / 2) * 2;
    const float c = cs[0], s = cs[1];
    const float q1 = q[(long)b * d + col], q2 = q[(long)b * d + col + 1];
    q[(long)b * d + col] = fmaf(q1, c, q2 * s);
    q[(long)b * d + col + 1] = fmaf(q2, c, -q1 * s);
    if (rotate_k) {
      const float r1 = fmaf(k1, c, k2 * s), r2 = fmaf(k2, c, -k1 * s);
      k1 = r1; k2 = r2;
    }
  }
  ET::store_two(K + b * bstride + (long)pos * d + col, k1, k2);
  if (vnew) ET::store_two(V + b * bstride + (long)pos * d + col, vnew[(long)b * d + col], vnew[(long)b * d + col + 1]);
}

__global__ __launch_bounds__(256) void zero_ints_kernel(int* __restrict__ p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}

// ------------------------------------------------------------------------------------------------
// vanilla K+V decode (flash-decoding layout): one wave per (b, split, head); 16 lanes span the
// head's d_k columns in 16-byte vectors (NPASS vectors per lane), the 4 lane groups take
// alternating rows with their own running (m, l, acc), merged at the end.
// ------------------------------------------------------------------------------------------------
template <class ET, int NPASS>
__global__ __launch_bounds__(256) void vanilla_kernel(
    const float* __restrict__ q, const typename ET::elem* __restrict__ K,
    const typename ET::elem* __restrict__ V, long bstride, const int32_t* __restrict__ seq_lens,
    int T, int H, int d_k, int nsplit, float scale, float* __restrict__ accp,
    float* __restrict__ mpart, float* __restrict__ lpart) {
  constexpr int VEC = ET::VEC;
  constexpr int UNR = 4;
  const int b = blockIdx.z, sp = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int h = blockIdx.x * 4 + wave;
  if (h >= H) return;
  const int idx = lane & 15, rg = lane >> 4;
  const int e = H * d_k;
  const int cph = d_k / VEC;                   // vectors per head row
  const int len = seq_len_of(seq_lens, b, T);
  const int ts = split_rows(len, nsplit);          // the splits are cut on the sequence's own length
  const int t0 = sp * ts;
  const int t1 = min(len, t0 + ts);

  float qv[NPASS][VEC];
  bool act[NPASS];
#pragma unroll
  for (int p = 0; p < NPASS; ++p) {
    act[p] = (p * 16 + idx) < cph;
#pragma unroll
    for (int j = 0; j < VEC; ++j)
      qv[p][j] = act[p] ? q[(long)b * e + h * d_k + (p * 16 + idx) * VEC + j] * scale : 0.f;
  }
  float m = NEG_INF, l = 0.f;
  float acc[NPASS][VEC];
#pragma unroll
  for (int p = 0; p < NPASS; ++p)
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[p][j] = 0.f;

  const typename ET::elem* Kb = K + b * bstride + h * d_k;
  const typename ET::elem* Vb = V + b * bstride + h * d_k;

  for (int tb = t0 + rg; tb < t1; tb += 4 * UNR) {
    float kv[UNR][NPASS][VEC], vv[UNR][NPASS][VEC];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int t = min(tb + u * 4, t1 - 1);
#pragma unroll
      for (int p = 0; p < NPASS; ++p) {
        if (act[p]) {
          ET::load_stream(Kb + (long)t * e + (p * 16 + idx) * VEC, kv[u][p]);
          ET::load_stream(Vb + (long)t * e + (p * 16 + idx) * VEC, vv[u][p]);
        } else {
#pragma unroll
          for (int j = 0; j < VEC; ++j) kv[u][p][j] = vv[u][p][j] = 0.f;
        }
      }
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      float s = 0.f;
#pragma unroll
      for (int p = 0; p < NPASS; ++p)
#pragma unroll
        for (int j = 0; j < VEC; ++j) s = fmaf(qv[p][j], kv[u][p][j], s);
      s += __shfl_xor(s, 1);
      s += __shfl_xor(s, 2);
      s += __shfl_xor(s, 4);
      s += __shfl_xor(s, 8);
      const bool ok = (tb + u * 4) < t1;
      if (ok) {
        const float mn = fmaxf(m, s);
        const float alpha = __expf(m - mn);      // m = -inf first time: exp(-inf) = 0
        const float pw = __expf(s - mn);
        l = l * alpha + pw;
#pragma unroll
        for (int p = 0; p < NPASS; ++p)
#pragma unroll
          for (int j = 0; j < VEC; ++j) acc[p][j] = fmaf(pw, vv[u][p][j], acc[p][j] * alpha);
        m = mn;
      }
    }
  }
  // merge the 4 row groups (lanes idx, idx+16, idx+32, idx+48)
  float mall = fmaxf(m, __shfl_xor(m, 16));
  mall = fmaxf(mall, __shfl_xor(mall, 32));
  const float w = (m == NEG_INF) ? 0.f : __expf(m - mall);
  l *= w;
  l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
#pragma unroll
  for (int p = 0; p < NPASS; ++p)
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      float a = acc[p][j] * w;
      a += __shfl_xor(a, 16);
      a += __shfl_xor(a, 32);
      acc[p][j] = a;
    }
  const long pb = ((long)b * nsplit + sp) * H + h;
  if (lane == 0) { mpart[pb] = mall; lpart[pb] = l; }
  if (rg == 0) {
#pragma unroll
    for (int p = 0; p < NPASS; ++p)
      if (act[p]) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) accp[pb * d_k + (p * 16 + idx) * VEC + j] = acc[p][j];
      }
  }
}

// ------------------------------------------------------------------------------------------------
// vanilla K+V decode, bf16, packed lanes: every lane of a wave carries live columns and a wave's
// piece of a cache row is a whole number of 128-byte lines, whatever the head width:
//   d_k = 128, 64, 32, 16, 8: a lane holds 8 columns (16 bytes); a head spans LPH = d_k / 8 lanes and
//     16 / LPH neighbouring heads share a 16-lane group (256 bytes of the row), four rows per load;
//   d_k = 96: a lane holds 6 columns (12 bytes), a head spans 16 lanes and two neighbouring heads
//     make 32 lanes (384 bytes = three lines), two rows per load.
// Each group of lanes that shares rows keeps its own running (reference, sum, accumulator) in the log2
// domain (the reference moves only when the maximum has grown by more than 2^6, as in the slim kernels)
// and the groups are merged at the end.  The context splits are cut on the sequence's own length.
// ------------------------------------------------------------------------------------------------
typedef unsigned vu3 __attribute__((ext_vector_type(3)));
typedef unsigned vu4 __attribute__((ext_vector_type(4)));
typedef __bf16 vbf2 __attribute__((ext_vector_type(2)));

template <int CTRL>
__device__ __forceinline__ float vdpp_add(float v) {
  return v + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

template <int CPL, int LPH>
__global__ __launch_bounds__(256) void vanilla_packed_kernel(
    const float* __restrict__ q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V, long bstride,
    const int32_t* __restrict__ seq_lens, int T, int H, int d_k, int nsplit, float scale_log2,
    float* __restrict__ accp, float* __restrict__ mpart, float* __restrict__ lpart) {
  constexpr int HPW = (CPL == 6) ? 2 : 16 / LPH;      // heads of a wave
  constexpr int LR = LPH * HPW;                       // lanes per cache row: 16 or 32
  constexpr int RG = 64 / LR;                         // rows per load
  constexpr int UNR = 16 / RG;                        // loads of K (and of V) in flight: 16 rows per wave and round
  constexpr int NW = CPL / 2;                         // dwords per lane and row
  constexpr float SLACK = 6.0f;
  const int b = blockIdx.z, sp = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int h0 = (blockIdx.x * 4 + wave) * HPW;
  if (h0 >= H) return;
  const int lr = lane % LR, rg = lane / LR;
  const int h = h0 + lr / LPH, li = lr % LPH;
  const bool live = h < H;
  const int e = H * d_k;
  const int col = (live ? h : h0) * d_k + li * CPL;   // (heads past the end re-read the first head: weighted with a zero query)
  const int len = seq_len_of(seq_lens, b, T);
  const int ts = split_rows(len, nsplit);
  const int t0 = sp * ts;
  const int t1 = min(len, t0 + ts);

  // the query of this lane's columns, pre-scaled, as bf16 hi + lo pairs for the packed dot product
  unsigned qh[NW], ql[NW];
#pragma unroll
  for (int c = 0; c < NW; ++c) {
    const float f0 = live ? q[(long)b * e + col + 2 * c] * scale_log2 : 0.f;
    const float f1 = live ? q[(long)b * e + col + 2 * c + 1] * scale_log2 : 0.f;
    const __bf16 a0 = (__bf16)f0, a1 = (__bf16)f1;
    const vbf2 hi = {a0, a1};
    const vbf2 lo = {(__bf16)(f0 - (float)a0), (__bf16)(f1 - (float)a1)};
    qh[c] = __builtin_bit_cast(unsigned, hi);
    ql[c] = __builtin_bit_cast(unsigned, lo);
  }
  float m = NEG_INF, l = 0.f;
  float acc[CPL];
#pragma unroll
  for (int j = 0; j < CPL; ++j) acc[j] = 0.f;

  const char* Kb = reinterpret_cast<const char*>(K + b * bstride + col);
  const char* Vb = reinterpret_cast<const char*>(V + b * bstride + col);
  const size_t pitch = (size_t)e * 2;
  auto load = [&](const char* base, int t, unsigned (&r)[NW]) {
    if constexpr (CPL == 8) {
      const vu4 x = __builtin_nontemporal_load(reinterpret_cast<const vu4*>(base + (size_t)t * pitch));
#pragma unroll
      for (int c = 0; c < 4; ++c) r[c] = x[c];
    } else {
      typedef vu3 vu3_a4 __attribute__((aligned(4)));
      const vu3 x = __builtin_nontemporal_load(reinterpret_cast<const vu3_a4*>(base + (size_t)t * pitch));
#pragma unroll
      for (int c = 0; c < 3; ++c) r[c] = x[c];
    }
  };

  for (int tb = t0 + rg; tb < t1; tb += RG * UNR) {
    unsigned kr[UNR][NW], vr[UNR][NW];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int t = min(tb + u * RG, t1 - 1);          // rows past the end re-read the last row; they get no weight
      load(Kb, t, kr[u]);
      load(Vb, t, vr[u]);
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      float s0 = 0.f, s1 = 0.f;
#pragma unroll
      for (int c = 0; c < NW; ++c) {
        const unsigned kw = kr[u][c];
        const vbf2 kv = __builtin_bit_cast(vbf2, kw);
        s0 = __builtin_amdgcn_fdot2_f32_bf16(kv, __builtin_bit_cast(vbf2, qh[c]), s0, false);
        s1 = __builtin_amdgcn_fdot2_f32_bf16(kv, __builtin_bit_cast(vbf2, ql[c]), s1, false);
      }
      float s = s0 + s1;
      if (LPH > 1) s = vdpp_add<0xB1>(s);              // lane ^ 1
      if (LPH > 2) s = vdpp_add<0x4E>(s);              // lane ^ 2
      if (LPH > 4) s = vdpp_add<0x141>(s);             // other quad of the 8-lane half
      if (LPH > 8) s = vdpp_add<0x140>(s);             // other half of the 16-lane row
      const bool ok = (tb + u * RG) < t1;
      const float mn = (ok && s > m + SLACK) ? s : m;
      if (__any(mn != m)) {                            // the reference of some head moved: rescale (rare)
        const float alpha = __builtin_amdgcn_exp2f(m - mn);   // 1 where it did not move, 0 the first time
        l *= alpha;
#pragma unroll
        for (int j = 0; j < CPL; ++j) acc[j] *= alpha;
        m = mn;
      }
      const float pw = ok ? __builtin_amdgcn_exp2f(s - m) : 0.f;
      l += pw;
#pragma unroll
      for (int c = 0; c < NW; ++c) {
        acc[2 * c] = fmaf(pw, __uint_as_float(vr[u][c] << 16), acc[2 * c]);
        acc[2 * c + 1] = fmaf(pw, __uint_as_float(vr[u][c] & 0xffff0000u), acc[2 * c + 1]);
      }
    }
  }
  // merge the RG groups of lanes that walked different rows (lanes lr, lr + LR, ...)
  float mall = m;
  if (RG > 2) mall = fmaxf(mall, __shfl_xor(mall, 16));
  mall = fmaxf(mall, __shfl_xor(mall, 32));
  const float w = (m == NEG_INF) ? 0.f : __builtin_amdgcn_exp2f(m - mall);
  l *= w;
  if (RG > 2) l += __shfl_xor(l, 16);
  l += __shfl_xor(l, 32);
#pragma unroll
  for (int j = 0; j < CPL; ++j) {
    float a = acc[j] * w;
    if (RG > 2) a += __shfl_xor(a, 16);
    a += __shfl_xor(a, 32);
    acc[j] = a;
  }
  if (rg == 0 && live) {
    const long pb = ((long)b * nsplit + sp) * H + h;
    if (li == 0) { mpart[pb] = mall * 0.6931471805599453f; lpart[pb] = l; }   // (the merge kernel works with natural logarithms)
#pragma unroll
    for (int j = 0; j < CPL; ++j) accp[pb * d_k + li * CPL + j] = acc[j];
  }
}

__global__ __launch_bounds__(256) void vanilla_combine_kernel(const float* __restrict__ accp,
                                                              const float* __restrict__ mpart,
                                                              const float* __restrict__ lpart,
                                                              int nsplit, int H, int d_k,
                                                              float* __restrict__ out) {
  // one workgroup per (b, h): merge weights of the (<= 256) splits in LDS, then one thread per
  // output column sums the weighted partial accumulators with independent loads
  __shared__ float wgt[256];
  __shared__ float red[256];
  const int b = blockIdx.y, h = blockIdx.x, tid = threadIdx.x;
  const long pb0 = ((long)b * nsplit) * H + h;
  const float ms = tid < nsplit ? mpart[pb0 + (long)tid * H] : NEG_INF;
  red[tid] = ms;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) red[tid] = fmaxf(red[tid], red[tid + o]);
    __syncthreads();
  }
  const float m = red[0];
  __syncthreads();
  const float w = (ms == NEG_INF) ? 0.f : __expf(ms - m);
  wgt[tid] = w;
  red[tid] = tid < nsplit ? w * lpart[pb0 + (long)tid * H] : 0.f;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (tid < o) red[tid] += red[tid + o];
    __syncthreads();
  }
  const float inv = 1.f / red[0];
  for (int j = tid; j < d_k; j += 256) {
    float num = 0.f;
    int s = 0;
    for (; s + 8 <= nsplit; s += 8) {
      float v[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) v[q] = accp[(pb0 + (long)(s + q) * H) * d_k + j];
#pragma unroll
      for (int q = 0; q < 8; ++q) num = fmaf(wgt[s + q], v[q], num);
    }
    for (; s < nsplit; ++s) num = fmaf(wgt[s], accp[(pb0 + (long)s * H) * d_k + j], num);
    out[((long)b * H + h) * d_k + j] = num * inv;
  }
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
void launch_head_scores(int dtype, const float* q, long q_bstride, const void* M, long m_bstride,
                        long row_pitch, const int32_t* rows_per_b, int rows, int e, int H, int d_k,
                        float scale, float* S, long s_bstride, const float* rope, int B, hipStream_t st) {
  dim3 grid((rows + HS_ROWS - 1) / HS_ROWS, B);
  const int nvec = e / vec_elems(dtype);
  const size_t smem = sizeof(float) * ((size_t)e + 4 * (size_t)nvec);
  if (dtype == DT_BF16) {
    (void)hipFuncSetAttribute((const void*)head_scores_kernel<BF16>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    hipLaunchKernelGGL(head_scores_kernel<BF16>, grid, dim3(256), smem, st, q, q_bstride,
                       (const uint16_t*)M, m_bstride, row_pitch, rows_per_b, rows, e, H, d_k, scale, S, s_bstride, rope);
  } else {
    (void)hipFuncSetAttribute((const void*)head_scores_kernel<F32>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    hipLaunchKernelGGL(head_scores_kernel<F32>, grid, dim3(256), smem, st, q, q_bstride,
                       (const float*)M, m_bstride, row_pitch, rows_per_b, rows, e, H, d_k, scale, S, s_bstride, rope);
  }
}

void launch_dense_scores(int dtype, const float* qt, const void* X, long x_bstride, int d_model,
                         const int32_t* seq_lens, int T, int H, float scale, float* S, int B,
                         hipStream_t st) {
  dim3 grid((T + DS_T - 1) / DS_T, (H + DS_H - 1) / DS_H, B);
  if (dtype == DT_BF16)
    hipLaunchKernelGGL(dense_scores_kernel<BF16>, grid, dim3(256), 0, st, qt, (const uint16_t*)X,
                       x_bstride, d_model, seq_lens, T, H, scale, S);
  else
    hipLaunchKernelGGL(dense_scores_kernel<F32>, grid, dim3(256), 0, st, qt, (const float*)X,
                       x_bstride, d_model, seq_lens, T, H, scale, S);
}

void launch_weighted_sum(int dtype, const float* S, const void* M, long m_bstride, int width,
                         const int32_t* seq_lens, int T, int H, int nsplit, float* Cpart,
                         float* mpart, float* lpart, int B, hipStream_t st) {
  const int ncolblk = (width + WS_COLS - 1) / WS_COLS;
  const int nhb = (H + WS_HB - 1) / WS_HB;
  dim3 grid(ncolblk * nhb, nsplit, B);
  if (dtype == DT_BF16)
    hipLaunchKernelGGL(weighted_sum_kernel<BF16>, grid, dim3(256), 0, st, S, (const uint16_t*)M,
                       m_bstride, width, seq_lens, T, H, nsplit, ncolblk, Cpart, mpart, lpart);
  else
    hipLaunchKernelGGL(weighted_sum_kernel<F32>, grid, dim3(256), 0, st, S, (const float*)M,
                       m_bstride, width, seq_lens, T, H, nsplit, ncolblk, Cpart, mpart, lpart);
}

void launch_combine(const float* Cpart, const float* mpart, const float* lpart, int nsplit, int H,
                    int width, float* Cn, int B, hipStream_t st) {
  dim3 grid((unsigned)(((long)H * width + 255) / 256), B);
  hipLaunchKernelGGL(combine_kernel, grid, dim3(256), 0, st, Cpart, mpart, lpart, nsplit, H, width, Cn);
}

void launch_project(int dtype, const float* Cn, const void* W, int rows, int e, int H, int d_k,
                    float* out, int B, hipStream_t st) {
  dim3 grid((e + 63) / 64, (B + 3) / 4);
  if (dtype == DT_BF16)
    hipLaunchKernelGGL(project_kernel<BF16>, grid, dim3(PROJ_WAVES * 64), 0, st, Cn, (const uint16_t*)W, rows, e, H, d_k, out, B);
  else
    hipLaunchKernelGGL(project_kernel<F32>, grid, dim3(PROJ_WAVES * 64), 0, st, Cn, (const float*)W, rows, e, H, d_k, out, B);
}

void launch_append(int dtype, const float* knew, const float* vnew, void* K, void* V, long bstride,
                   const int32_t* seq_lens, int T, int d, int d_k, const float* rope, float* q, int rotate_k,
                   int B, hipStream_t st) {
  dim3 grid((d / 2 + 255) / 256, B);
  if (dtype == DT_BF16)
    hipLaunchKernelGGL(append_kernel<BF16>, grid, dim3(256), 0, st, knew, vnew, (uint16_t*)K, (uint16_t*)V,
                       bstride, seq_lens, T, d, d_k, rope, q, rotate_k);
  else
    hipLaunchKernelGGL(append_kernel<F32>, grid, dim3(256), 0, st, knew, vnew, (float*)K, (float*)V,
                       bstride, seq_lens, T, d, d_k, rope, q, rotate_k);
}

void launch_zero_ints(int* p, int n, hipStream_t st) {
  hipLaunchKernelGGL(zero_ints_kernel, dim3((n + 255) / 256), dim3(256), 0, st, p, n);
}

// heads a wave of the packed bf16 kernel covers (0: this head width takes the plain kernel)
int vanilla_heads_per_wave(int dtype, int d_k) {
  if (dtype != DT_BF16) return 0;
  if (d_k == 96) return 2;
  if (d_k == 8 || d_k == 16 || d_k == 32 || d_k == 64 || d_k == 128) return 128 / d_k;
  return 0;
}

void launch_vanilla(int dtype, const float* q, const void* K, const void* V, long bstride,
                    const int32_t* seq_lens, int T, int H, int d_k, int nsplit, float* acc,
                    float* mpart, float* lpart, float* out, int B, hipStream_t st) {
  const float scale = 1.0f / sqrtf((float)d_k);
  const int cph = d_k / vec_elems(dtype);
  if (const int hpw = vanilla_heads_per_wave(dtype, d_k)) {
    dim3 grid(((H + hpw - 1) / hpw + 3) / 4, nsplit, B);
    const float sl2 = scale * 1.4426950408889634f;
    auto go = [&](auto cpl, auto lph) {
      hipLaunchKernelGGL((vanilla_packed_kernel<decltype(cpl)::value, decltype(lph)::value>), grid, dim3(256), 0, st, q,
                         (const uint16_t*)K, (const uint16_t*)V, bstride, seq_lens, T, H, d_k, nsplit, sl2, acc, mpart, lpart);
    };
    using C8 = std::integral_constant<int, 8>;
    switch (d_k) {
      case 96: go(std::integral_constant<int, 6>{}, std::integral_constant<int, 16>{}); break;
      case 128: go(C8{}, std::integral_constant<int, 16>{}); break;
      case 64: go(C8{}, std::integral_constant<int, 8>{}); break;
      case 32: go(C8{}, std::integral_constant<int, 4>{}); break;
      case 16: go(C8{}, std::integral_constant<int, 2>{}); break;
      default: go(C8{}, std::integral_constant<int, 1>{}); break;
    }
  } else {
  dim3 grid((H + 3) / 4, nsplit, B);
  if (dtype == DT_BF16) {
    if (cph <= 16)
      hipLaunchKernelGGL((vanilla_kernel<BF16, 1>), grid, dim3(256), 0, st, q, (const uint16_t*)K,
                         (const uint16_t*)V, bstride, seq_lens, T, H, d_k, nsplit, scale, acc, mpart, lpart);
    else
      hipLaunchKernelGGL((vanilla_kernel<BF16, 2>), grid, dim3(256), 0, st, q, (const uint16_t*)K,
                         (const uint16_t*)V, bstride, seq_lens, T, H, d_k, nsplit, scale, acc, mpart, lpart);
  } else {
    if (cph <= 16)
      hipLaunchKernelGGL((vanilla_kernel<F32, 1>), grid, dim3(256), 0, st, q, (const float*)K,
                         (const float*)V, bstride, seq_lens, T, H, d_k, nsplit, scale, acc, mpart, lpart);
    else
      hipLaunchKernelGGL((vanilla_kernel<F32, 2>), grid, dim3(256), 0, st, q, (const float*)K,
                         (const float*)V, bstride, seq_lens, T, H, d_k, nsplit, scale, acc, mpart, lpart);
  }
  }
  dim3 g2(H, B);
  hipLaunchKernelGGL(vanilla_combine_kernel, g2, dim3(256), 0, st, acc, mpart, lpart, nsplit, H, d_k, out);
}

// ---- measurement helper: a plain streaming read -------------------------------------------------
namespace {
__global__ __launch_bounds__(256) void read_probe_kernel(const uint4* __restrict__ p, size_t n16, unsigned* sink) {
  // each workgroup walks a contiguous chunk with eight 16-byte loads in flight per thread
  const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t lo = per * blockIdx.x, hi = lo + per < n16 ? lo + per : n16;
  unsigned acc = 0;
  size_t i = lo + threadIdx.x;
  for (; i + 7 * 256 < hi; i += 8 * 256) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = p[i + u * 256];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < hi; i += 256) { const uint4 v = p[i]; acc ^= v.x ^ v.y ^ v.z ^ v.w; }
  if (acc == 0x9e3779b9u && sink) *sink = acc;        // (keeps the loads alive; practically never taken)
}
}  // namespace

void launch_read_probe(const void* buf, size_t bytes, hipStream_t st) {
  hipLaunchKernelGGL(read_probe_kernel, dim3(16384), dim3(256), 0, st, (const uint4*)buf, bytes / 16, (unsigned*)nullptr);
}

}  // namespace slim
