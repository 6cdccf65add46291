// bf16 fast path of the X-cache scheme for projection width e > d_model (non-square section,
// Fig. 4): the cache holds the layer input X [T][d_model]; K and V are never formed.
//
//   xq_tilde_kernel   : q~_h = q_h W_K,h^T           [B][H][d_model]   (W_K read once)
//   xscores_kernel    : s[h][t] = q~_h . X[t]        [B][H][T], log2 domain, on MFMA
//   xweighted_kernel  : per context split, m = max s, l = sum 2^(s-m), C_h = sum_t 2^(s-m) X[t]
//                       on MFMA, one contraction for 32 heads at a time
// followed by the merge + projection of the K-cache path with W_V in place of W_KV.
//
// All heads use the full row of X here (no per-head column slice), so the scores are a plain
// dense product over d_model; they are written out (H x T x 4 bytes per sequence, small next to the
// 2 x e-wide caches the scheme avoids) and the weighted sum is a second pass over X.
#include "slim_kernels.h"

#include <math.h>

namespace slim {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr float NEG_INF = -INFINITY;

__device__ __forceinline__ int seq_len_of(const int32_t* lens, int b, int T) {
  if (!lens) return T;
  const int n = lens[b];
  return n < 0 ? 0 : (n > T ? T : n);
}

// 8 fp32 values -> bf16 hi and bf16 lo (x = hi + lo up to 2^-17 relative)
__device__ __forceinline__ void split_hi_lo(const float (&x)[8], bf16x8& hi, bf16x8& lo) {
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const __bf16 h = (__bf16)x[j];
    hi[j] = h;
    lo[j] = (__bf16)(x[j] - (float)h);
  }
}

// 8 rows x 8 bf16 columns per lane  ->  8 operands (one per column), each 8 rows of that column.
__device__ __forceinline__ void transpose8x8(const u32x4 (&kt)[8], u32x4 (&a)[8]) {
#pragma unroll
  for (int jp = 0; jp < 4; ++jp) {
    const u32x4 lo = kt[2 * jp], hi = kt[2 * jp + 1];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      a[2 * c][jp] = __builtin_amdgcn_perm(hi[c], lo[c], 0x05040100u);
      a[2 * c + 1][jp] = __builtin_amdgcn_perm(hi[c], lo[c], 0x07060302u);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// q~[b][h][c] = sum_j q[b][h d_k + j] W_K[c][h d_k + j]
// grid (H / XQ_HEADS, d_model / 128, batch chunks of 16); a wave owns 16 rows c of W_K for XQ_HEADS heads.
// MFMA: A = W_K block (M = 16 rows c, K = the head's columns j), B = q^T (N = sequences) as hi + lo.
// ------------------------------------------------------------------------------------------------
constexpr int XQ_HEADS = 4;

__global__ __launch_bounds__(512) void xq_tilde_kernel(const float* q, const uint16_t* Wk, float* qt, int B,
                                                       int H, int d_k, int dm, int e, int* counters, int ncounters) {
  // (the arrival counters of the projection that ends this call start at 0)
  if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)
    for (int i = threadIdx.x; i < ncounters; i += 512) counters[i] = 0;
  const int bbase = blockIdx.z * 16;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int n = lane & 15, kq = lane >> 4;
  const int c0 = (blockIdx.y * 8 + w) * 16;
  if (c0 >= dm) return;
  const int b = bbase + n;
  const int nks = d_k / 32;                            // 1..4 k-steps per head
  // XQ_HEADS heads per wave: all their loads of W_K are issued before the first MFMA
  u32x4 av[XQ_HEADS][4];
#pragma unroll
  for (int hh = 0; hh < XQ_HEADS; ++hh) {
    const int h = min(blockIdx.x * XQ_HEADS + hh, H - 1);
    const uint16_t* wrow = Wk + (size_t)(c0 + n) * e + (size_t)h * d_k + kq * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) av[hh][ks] = *reinterpret_cast<const u32x4*>(wrow + min(ks, nks - 1) * 32);
  }
#pragma unroll
  for (int hh = 0; hh < XQ_HEADS; ++hh) {
    const int h = blockIdx.x * XQ_HEADS + hh;
    if (h >= H) break;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if (ks >= nks) break;
      float x[8];
      const float* qsrc = q + (size_t)min(b, B - 1) * e + (size_t)h * d_k + ks * 32 + kq * 8;
      const f32x4 lo4 = *reinterpret_cast<const f32x4*>(qsrc), hi4 = *reinterpret_cast<const f32x4*>(qsrc + 4);
#pragma unroll
      for (int j = 0; j < 4; ++j) { x[j] = (b < B) ? lo4[j] : 0.f; x[4 + j] = (b < B) ? hi4[j] : 0.f; }
      bf16x8 hi, lo;
      split_hi_lo(x, hi, lo);
      const bf16x8 a8 = __builtin_bit_cast(bf16x8, av[hh][ks]);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8, hi, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8, lo, acc, 0, 0, 0);
    }
    // D: column n = sequence, rows kq*4 + r = c0 + ...
    if (b < B) *reinterpret_cast<f32x4*>(qt + ((size_t)b * H + h) * dm + c0 + kq * 4) = acc;
  }
}

// ------------------------------------------------------------------------------------------------
// s[b][h][t] = scale * sum_c X[b][t][c] q~[b][h][c]       (scale = log2(e) / sqrt(d_k))
// grid (row chunks of nblk x 256, ceil(H / HG), B), HG = 16 HT heads per workgroup (HT = 2 unless q~ of 32
// heads does not fit LDS).  The workgroup keeps q~ of its heads in LDS as bf16 hi + lo (B operands); a wave
// owns 32 rows of X per block (A operands straight from global memory).
// ------------------------------------------------------------------------------------------------
constexpr int XS_PAD = 8;   // bf16 elements of padding per q~ row in LDS (spreads the rows over the banks)
constexpr size_t XS_LDS_MAX = 150 * 1024;

template <int HT>
__global__ __launch_bounds__(512) void xscores_kernel(const float* qt, const uint16_t* X, long x_bstride,
                                                      const int32_t* seq_lens, int T, int H, int dm, float scale,
                                                      float* S, int nblk) {
  extern __shared__ __align__(16) uint16_t qs[];                    // [2][HG][dm + XS_PAD]
  constexpr int HG = 16 * HT;
  const int b = blockIdx.z, hg = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int n = lane & 15, kq = lane >> 4;
  const int pitch = dm + XS_PAD;
  const int len = seq_len_of(seq_lens, b, T);
  const int row_base = blockIdx.x * nblk * 256;       // this workgroup: nblk blocks of 256 rows
  if (row_base >= len) return;                        // (workgroup-uniform) nothing to score here
  {
    const int dm8 = dm >> 3;
    for (int v = tid; v < HG * dm8; v += 512) {       // 8 columns per item
      const int hd = v / dm8, c = (v - hd * dm8) * 8;
      const int h = hg * HG + hd;
      float x[8];
      if (h < H) {
        const float* src = qt + ((size_t)b * H + h) * dm + c;
        const f32x4 lo4 = *reinterpret_cast<const f32x4*>(src), hi4 = *reinterpret_cast<const f32x4*>(src + 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) { x[j] = lo4[j] * scale; x[4 + j] = hi4[j] * scale; }
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) x[j] = 0.f;
      }
      bf16x8 hi, lo;
      split_hi_lo(x, hi, lo);
      *reinterpret_cast<bf16x8*>(&qs[hd * pitch + c]) = hi;
      *reinterpret_cast<bf16x8*>(&qs[(HG + hd) * pitch + c]) = lo;
    }
  }
  __syncthreads();
  const int nks = dm / 32;                             // a multiple of 4
  const uint16_t* Xb = X + (size_t)b * x_bstride + kq * 8;
  // A wave owns 32 rows of a 256-row block (two A operands share every B operand read from LDS);
  // 8 k-steps (256 columns) of A operands per buffer, the other buffer is in flight meanwhile.
  constexpr int KH = 8;
  u32x4 a0[2][KH], a1[2][KH];
  auto load_part = [&](u32x4 (&a)[2][KH], int blk, int kbase) {
    const int t0 = row_base + blk * 256 + w * 32;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      const uint16_t* xrow = Xb + (size_t)min(t0 + rb * 16 + n, len - 1) * dm;
#pragma unroll
      for (int u = 0; u < KH; ++u) a[rb][u] = *reinterpret_cast<const u32x4*>(xrow + min(kbase + u, nks - 1) * 32);
    }
  };
  auto mma_part = [&](const u32x4 (&a)[2][KH], int kbase, f32x4 (&acc)[2][HT]) {
#pragma unroll
    for (int u = 0; u < KH; ++u) {
      if (kbase + u >= nks) break;
      const int coff = (kbase + u) * 32 + kq * 8;
#pragma unroll
      for (int ht = 0; ht < HT; ++ht) {
        const bf16x8 bh = *reinterpret_cast<const bf16x8*>(&qs[(ht * 16 + n) * pitch + coff]);
        const bf16x8 bl = *reinterpret_cast<const bf16x8*>(&qs[(HG + ht * 16 + n) * pitch + coff]);
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
          const bf16x8 a8 = __builtin_bit_cast(bf16x8, a[rb][u]);
          acc[rb][ht] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8, bh, acc[rb][ht], 0, 0, 0);
          acc[rb][ht] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8, bl, acc[rb][ht], 0, 0, 0);
        }
      }
    }
  };
  const int nparts = (nks + KH - 1) / KH;              // parts per block
  const int nb_here = min(nblk, (len - row_base + 255) / 256);
  const int total = nb_here * nparts;                  // parts this wave goes through
  f32x4 acc[2][HT];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int ht = 0; ht < HT; ++ht) acc[rb][ht] = f32x4{0.f, 0.f, 0.f, 0.f};
  auto flush = [&](int part) {                         // last part of a block: write its scores
    if ((part + 1) % nparts != 0) return;
    const int t0 = row_base + (part / nparts) * 256 + w * 32;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int ht = 0; ht < HT; ++ht) {
        const int h = hg * HG + ht * 16 + n;           // D: column n = head, rows kq*4 + r
        if (h < H) {
          float* dst = S + ((size_t)b * H + h) * T + t0 + rb * 16 + kq * 4;
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (t0 + rb * 16 + kq * 4 + r < len) dst[r] = acc[rb][ht][r];
        }
        acc[rb][ht] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
  };
  load_part(a0, 0, 0);
  for (int i = 0; i < total; i += 2) {                 // even parts in a0, odd parts in a1
    if (i + 1 < total) load_part(a1, (i + 1) / nparts, ((i + 1) % nparts) * KH);
    mma_part(a0, (i % nparts) * KH, acc);
    flush(i);
    if (i + 2 < total) load_part(a0, (i + 2) / nparts, ((i + 2) % nparts) * KH);
    if (i + 1 < total) {
      mma_part(a1, ((i + 1) % nparts) * KH, acc);
      flush(i + 1);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Weighted sum of the rows of X for one (sequence, context split, group of 32 heads, block of
// 1024 columns): wave w owns columns [128 w, 128 w + 128) of the block and all rows of the split.
// Register tile and MFMA layout as in the K-cache stream kernel: lane (idx = l % 16, rg = l / 16)
// loads 16 bytes of rows rg*8 .. rg*8+7, transposes its 8x8 block into 8 A operands; B = weights
// P^T (lane (n = head, kg = row group) reads 8 consecutive scores of head n).
// Writes Cpart[(b nsplit + s)][h][c] (unnormalised), mpart (log2 domain) and lpart.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(512) void xweighted_kernel(const float* S, const uint16_t* X, long x_bstride,
                                                        const int32_t* seq_lens, int T, int H, int dm, int nsplit,
                                                        float* Cpart, float* mpart, float* lpart) {
  constexpr int NT = 2;
  const int b = blockIdx.z, s = blockIdx.x;
  const int nhg = (H + 31) / 32;
  const int hg = blockIdx.y % nhg, cb = blockIdx.y / nhg;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int idx = lane & 15, rg = lane >> 4;
  const int n = idx, kg = rg;
  const int col0 = cb * 1024 + w * 128;
  if (col0 >= dm) return;
  const int len = seq_len_of(seq_lens, b, T);
  const int rows_per = ((len + nsplit - 1) / nsplit + 31) / 32 * 32;
  const int r_lo = s * rows_per, r_hi = min(len, r_lo + rows_per);
  const int pid = b * nsplit + s;

  float m[NT];
  f32x4 acc[8][NT], accl[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    m[t] = NEG_INF;
    accl[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i][t] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const uint16_t* Xb = X + (size_t)b * x_bstride + col0 + idx * 8;
  auto load_tile = [&](u32x4 (&t)[8], int r0) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int r = min(r0 + rg * 8 + j, len - 1);     // rows past the end weigh nothing (masked below)
      t[j] = *reinterpret_cast<const u32x4*>(Xb + (size_t)r * dm);   // (re-read by the other head groups: keep it cached)
    }
  };
  // scores of a tile: lane (n, kg) takes rows r0 + kg*8 .. +7 of heads hg*32 + t*16 + n
  const bool vec_ok = (T % 4) == 0;                  // 16-byte aligned rows of S
  auto load_scores = [&](float (&x)[NT][8], int r0) {
    const int row = r0 + kg * 8;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int h = hg * 32 + t * 16 + n;
      const float* src = S + ((size_t)b * H + min(h, H - 1)) * T + row;
      if (h < H && row + 8 <= r_hi && vec_ok) {
        const f32x4 lo4 = *reinterpret_cast<const f32x4*>(src), hi4 = *reinterpret_cast<const f32x4*>(src + 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) { x[t][j] = lo4[j]; x[t][4 + j] = hi4[j]; }
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) x[t][j] = (h < H && row + j < r_hi) ? src[j] : NEG_INF;
      }
    }
  };
  u32x4 cur[8], nxt[8];
  float sx[NT][8], sn[NT][8];
  if (r_lo < r_hi) { load_tile(cur, r_lo); load_scores(sx, r_lo); }
  for (int r0 = r_lo; r0 < r_hi; r0 += 32) {
    const bool more = r0 + 32 < r_hi;
    if (more) { load_tile(nxt, r0 + 32); load_scores(sn, r0 + 32); }
    bf16x8 pb[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      float (&x)[8] = sx[t];
      float tmax = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
      const float mn = fmaxf(m[t], tmax);
      const float ref = (mn == NEG_INF) ? 0.f : mn;
      const float alpha = __builtin_amdgcn_exp2f(m[t] - ref);
#pragma unroll
      for (int j = 0; j < 8; ++j) pb[t][j] = (__bf16)__builtin_amdgcn_exp2f(x[j] - ref);
      m[t] = mn;
      if (__any(alpha != 1.f)) {
        accl[t] *= alpha;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i][t] *= alpha;
      }
    }
    u32x4 am[8];
    transpose8x8(cur, am);
    const u32x4 ones_bits = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
    const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_bits);
#pragma unroll
    for (int t = 0; t < NT; ++t) accl[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[t], accl[t], 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bf16x8 av = __builtin_bit_cast(bf16x8, am[i]);
#pragma unroll
      for (int t = 0; t < NT; ++t)
        acc[i][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, pb[t], acc[i][t], 0, 0, 0);
    }
    if (more) {
#pragma unroll
      for (int j = 0; j < 8; ++j) cur[j] = nxt[j];
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int j = 0; j < 8; ++j) sx[t][j] = sn[t][j];
    }
  }
  // acc[i][t][r]: column col0 + (rg*4 + r)*8 + i, head hg*32 + t*16 + n
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int h = hg * 32 + t * 16 + n;
    if (h >= H) continue;
    float* dst = Cpart + ((size_t)pid * H + h) * dm + col0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int c = (rg * 4 + r) * 8;
      f32x4 lo4, hi4;
#pragma unroll
      for (int i = 0; i < 4; ++i) { lo4[i] = acc[i][t][r]; hi4[i] = acc[4 + i][t][r]; }
      *reinterpret_cast<f32x4*>(dst + c) = lo4;
      *reinterpret_cast<f32x4*>(dst + c + 4) = hi4;
    }
    if (cb == 0 && w == 0 && kg == 0) {
      mpart[(size_t)pid * H + h] = m[t];
      lpart[(size_t)pid * H + h] = accl[t][0];
    }
  }
}

}  // namespace

bool xcache_fast_ok(int dtype, int H, int d_model, int d_k) {
  return dtype == DT_BF16 && d_model % 128 == 0 && d_k % 32 == 0 && d_k >= 32 && H >= 1 &&
         (size_t)2 * 16 * (d_model + XS_PAD) * 2 <= XS_LDS_MAX;
}

int xcache_splits(int B, int H, int T, int d_model) {
  const int per = B * ((H + 31) / 32) * ((d_model + 1023) / 1024);
  int s = (256 + per - 1) / per;
  const int cap = (T + 127) / 128;
  if (s > cap) s = cap;
  if (s > PROJ_MAX_PARTS) s = PROJ_MAX_PARTS;
  return s < 1 ? 1 : s;
}

void launch_xq_tilde(const float* q, const void* Wk, float* qt, int B, int H, int d_k, int d_model, int e,
                     int* counters, int ncounters, hipStream_t st) {
  dim3 grid((H + XQ_HEADS - 1) / XQ_HEADS, (d_model + 127) / 128, (B + 15) / 16);
  hipLaunchKernelGGL(xq_tilde_kernel, grid, dim3(512), 0, st, q, (const uint16_t*)Wk, qt, B, H, d_k, d_model, e,
                     counters, ncounters);
}

void launch_xscores(const float* qt, const void* X, long x_bstride, const int32_t* seq_lens, int T, int H,
                    int d_model, float scale, float* S, int B, hipStream_t st) {
  // 32 heads per workgroup when their q~ fits LDS (and there are more than 16), else 16
  const bool wide = H > 16 && (size_t)2 * 32 * (d_model + XS_PAD) * sizeof(uint16_t) <= XS_LDS_MAX;
  const int HG = wide ? 32 : 16;
  // blocks of 256 rows per workgroup: about one workgroup per CU (the q~ operands are staged per workgroup)
  const int blocks = (T + 255) / 256, per = ((H + HG - 1) / HG) * B;
  int nblk = (blocks * per + 255) / 256;
  if (nblk < 1) nblk = 1;
  dim3 grid((blocks + nblk - 1) / nblk, (H + HG - 1) / HG, B);
  const size_t lds = (size_t)2 * HG * (d_model + XS_PAD) * sizeof(uint16_t);
  static bool raised = false;
  if (!raised) {
    (void)hipFuncSetAttribute((const void*)xscores_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)XS_LDS_MAX);
    (void)hipFuncSetAttribute((const void*)xscores_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)XS_LDS_MAX);
    raised = true;
  }
  if (wide)
    hipLaunchKernelGGL(xscores_kernel<2>, grid, dim3(512), lds, st, qt, (const uint16_t*)X, x_bstride, seq_lens, T, H,
                       d_model, scale, S, nblk);
  else
    hipLaunchKernelGGL(xscores_kernel<1>, grid, dim3(512), lds, st, qt, (const uint16_t*)X, x_bstride, seq_lens, T, H,
                       d_model, scale, S, nblk);
}

void launch_xweighted(const float* S, const void* X, long x_bstride, const int32_t* seq_lens, int T, int H,
                      int d_model, int nsplit, float* Cpart, float* mpart, float* lpart, int B, hipStream_t st) {
  dim3 grid(nsplit, ((H + 31) / 32) * ((d_model + 1023) / 1024), B);
  hipLaunchKernelGGL(xweighted_kernel, grid, dim3(512), 0, st, S, (const uint16_t*)X, x_bstride, seq_lens, T, H,
                     d_model, nsplit, Cpart, mpart, lpart);
}

}  // namespace slim
