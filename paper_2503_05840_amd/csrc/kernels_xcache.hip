// bf16 fast path of the X-cache scheme (non-square section, Fig. 4; also the encoder-cache option of
// the encoder-decoder section): the cache holds the layer input X [T][d_model]; K and V are never formed.
//
//   xq_tilde_kernel   : q~_h = q_h W_K,h^T, scaled, as bf16 hi + lo in MFMA operand order (W_K read once)
//   xscores_kernel    : s[h][t] = q~_h . X[t]        [B][H][T padded to 32], log2 domain, on MFMA
//   xweighted_kernel  : per context split, m = reference, l = sum 2^(s-m), C_h = sum_t 2^(s-m) X[t]
//                       on MFMA, one contraction for 32 heads at a time
// followed by the merge + projection of the K-cache path with W_V in place of W_KV.
//
// All heads use the full row of X here (no per-head column slice), so the scores are a plain
// dense product over d_model; they are written out (H x T x 4 bytes per sequence, small next to the
// 2 x e-wide caches the scheme avoids) and the weighted sum is a second pass over X.
#include "slim_kernels.h"

#include "device_common.h"

namespace slim {
namespace {

// 8 fp32 values -> bf16 hi and bf16 lo (x = hi + lo up to 2^-17 relative)
__device__ __forceinline__ void split_hi_lo(const float (&x)[8], bf16x8& hi, bf16x8& lo) {
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const __bf16 h = (__bf16)x[j];
    hi[j] = h;
    lo[j] = (__bf16)(x[j] - (float)h);
  }
}

// Workgroup barrier for data exchanged through LDS only: waits for this wave's LDS operations, not for its
// global loads (__syncthreads() would also drain the tiles that are being prefetched from HBM).
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Workgroup i of a one-dimensional launch -> (unit, inner): a unit is a set of `ninner` workgroups that read
// the same data (a sequence's q~ or scores, the same rows of X).  Workgroups are dealt to the 8 XCDs round
// robin, each with an L2 of its own, so with `colocate` a unit's workgroups are the ones with the same
// i % 8 and consecutive i / 8: what they share is fetched into one L2 instead of up to eight.  (Where the
// dealing differs the mapping is still a bijection: only the sharing is lost.)  False: no such unit.
__device__ __forceinline__ bool unit_of_workgroup(int i, int ninner, int nunits, bool colocate, int& unit, int& inner) {
  if (colocate) {
    const int slot = i >> 3;
    unit = (slot / ninner) * 8 + (i & 7);
    inner = slot % ninner;
  } else {
    unit = i / ninner;
    inner = i % ninner;
  }
  return unit < nunits;
}

// ------------------------------------------------------------------------------------------------
// q~[b][h][c] = scale * sum_j q[b][h d_k + j] W_K[c][h d_k + j]   (scale = log2(e) / sqrt(d_k)), written
// as two bf16 arrays, hi = bf16(q~) and lo = bf16(q~ - hi), in the order the scores kernel's MFMA B operands
// take them: [b][tile of 16 heads][k-step of 32 columns][lane = (column / 8 % 4) * 16 + head % 16][8 columns],
// so that a wave reads one operand as 1 KB of consecutive bytes.
// grid (H / XQ_HEADS, d_model / 128, batch chunks of 16); a wave owns 16 rows c of W_K for XQ_HEADS heads.
// MFMA: A = W_K block (M = 16 rows c, K = the head's columns j), B = q^T (N = sequences) as hi + lo.
// The 8 waves share their B operands: the workgroup fetches its slice of q once (consecutive threads on
// consecutive floats), splits it and lays the operands out in LDS.  (Fetched per wave in operand order --
// a lane per sequence, rows of q 4 e bytes apart -- q cost more time than W_K: 16 lines per instruction that
// fall on few L2 channels, and every workgroup of a head asks for the same ones.)
// ------------------------------------------------------------------------------------------------
constexpr int XQ_HEADS = 4;
constexpr int XQ_QROW = 16 * 16 + 16;    // bytes per (head, k-step, k-group) of B operands in LDS: 16 sequences x 16 bytes + padding

__global__ __launch_bounds__(512) void xq_tilde_kernel(const float* q, const uint16_t* Wk, uint16_t* qt, int B,
                                                       int H, int d_k, int dm, int e, float scale, int* counters,
                                                       int ncounters) {
  __shared__ __align__(16) unsigned char qs[2][XQ_HEADS * 4 * 4 * XQ_QROW];   // hi, lo
  // (the arrival counters of the projection that ends this call start at 0)
  if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0)
    for (int i = threadIdx.x; i < ncounters; i += 512) counters[i] = 0;
  const int bbase = blockIdx.z * 16;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int n = lane & 15, kq = lane >> 4;
  const int c0 = (blockIdx.y * 8 + w) * 16;            // (d_model is a multiple of 128: every wave has rows)
  const int h0 = blockIdx.x * XQ_HEADS;
  const int b = bbase + n;
  const int nks = d_k / 32;                            // 1..4 k-steps per head
  // all loads of W_K are issued before anything else: they come from HBM
  u32x4 av[XQ_HEADS][4];
#pragma unroll
  for (int hh = 0; hh < XQ_HEADS; ++hh) {
    const int h = min(h0 + hh, H - 1);
    const uint16_t* wrow = Wk + (size_t)(c0 + n) * e + (size_t)h * d_k + kq * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) av[hh][ks] = *reinterpret_cast<const u32x4*>(wrow + min(ks, nks - 1) * 32);
  }
  // q of the workgroup's heads and sequences: 16 x XQ_HEADS d_k floats = nks pieces of 4 floats per thread
  {
    const int upq = d_k / 4;                           // pieces per head
    f32x4 qraw[4];
    int off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      qraw[i] = f32x4{0.f, 0.f, 0.f, 0.f};
      off[i] = 0;
      if (i < nks) {
        const int g = i * 512 + tid, bl = g / d_k, rem = g - bl * d_k, hh = rem / upq, j0 = (rem - hh * upq) * 4;
        // (heads past H and sequences past B: zeros)
        if (bbase + bl < B && h0 + hh < H)
          qraw[i] = *reinterpret_cast<const f32x4*>(q + (size_t)(bbase + bl) * e + (size_t)(h0 + hh) * d_k + j0);
        off[i] = ((hh * 4 + (j0 >> 5)) * 4 + ((j0 & 31) >> 3)) * XQ_QROW + bl * 16 + (j0 & 7) * 2;
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (i < nks) {
        unsigned hw[2], lw[2];
#pragma unroll
        for (int r = 0; r < 4; r += 2) {
          const float x0 = qraw[i][r], x1 = qraw[i][r + 1];
          const __bf16 hb0 = (__bf16)x0, hb1 = (__bf16)x1;
          const __bf16 l0 = (__bf16)(x0 - (float)hb0), l1 = (__bf16)(x1 - (float)hb1);
          hw[r / 2] = (unsigned)__builtin_bit_cast(uint16_t, hb0) | ((unsigned)__builtin_bit_cast(uint16_t, hb1) << 16);
          lw[r / 2] = (unsigned)__builtin_bit_cast(uint16_t, l0) | ((unsigned)__builtin_bit_cast(uint16_t, l1) << 16);
        }
        *reinterpret_cast<uint2*>(&qs[0][off[i]]) = make_uint2(hw[0], hw[1]);
        *reinterpret_cast<uint2*>(&qs[1][off[i]]) = make_uint2(lw[0], lw[1]);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int hh = 0; hh < XQ_HEADS; ++hh) {
    const int h = h0 + hh;
    if (h >= H) break;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if (ks < nks) {
        const int qo = ((hh * 4 + ks) * 4 + kq) * XQ_QROW + n * 16;
        const bf16x8 hi = *reinterpret_cast<const bf16x8*>(&qs[0][qo]);
        const bf16x8 lo = *reinterpret_cast<const bf16x8*>(&qs[1][qo]);
        const bf16x8 a8 = __builtin_bit_cast(bf16x8, av[hh][ks]);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8, hi, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8, lo, acc, 0, 0, 0);
      }
    }
    // D: column n = sequence, rows kq*4 + r = c0 + ...; stored scaled, as bf16 hi and lo halves
    if (b < B) {
      unsigned hw[2], lw[2];
#pragma unroll
      for (int r = 0; r < 4; r += 2) {
        const float x0 = acc[r] * scale, x1 = acc[r + 1] * scale;
        const __bf16 hb0 = (__bf16)x0, hb1 = (__bf16)x1;
        const __bf16 l0 = (__bf16)(x0 - (float)hb0), l1 = (__bf16)(x1 - (float)hb1);
        hw[r / 2] = (unsigned)__builtin_bit_cast(uint16_t, hb0) | ((unsigned)__builtin_bit_cast(uint16_t, hb1) << 16);
        lw[r / 2] = (unsigned)__builtin_bit_cast(uint16_t, l0) | ((unsigned)__builtin_bit_cast(uint16_t, l1) << 16);
      }
      // B-operand order of the scores kernel: [b][head tile][k-step of 32 columns][lane (kq, n)][8]
      const int c = c0 + kq * 4, nht = (H + 15) / 16;
      const size_t at = ((((size_t)b * nht + h / 16) * (dm / 32) + c / 32) * 64 + ((c % 32) / 8) * 16 + h % 16) * 8 + c % 8;
      *reinterpret_cast<uint2*>(qt + at) = make_uint2(hw[0], hw[1]);
      *reinterpret_cast<uint2*>(qt + (size_t)B * nht * 16 * dm + at) = make_uint2(lw[0], lw[1]);
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Both passes over X share one layout: a workgroup stages tiles of X in LDS with coalesced loads
// (every element of X leaves HBM once per pass) and its 8 waves split the HEADS: wave w owns head
// tile (16 heads) w % P of the P tiles in flight, P = 1, 2, 4 or 8, and shares the rest of the work
// with the 8 / P waves of the same head tile.  More than 16 P heads: several passes.
//
// xscores: s[b][h][t] = sum_c X[b][t][c] q~[b][h][c]   (log2 domain; q~ arrives scaled)
// grid (blocks of 128 rows, B).  X is staged in chunks of 256 columns (double-buffered: the next chunk
// travels HBM -> registers while this one is used, then registers -> LDS).  Per chunk a wave holds the
// B operands of its head tile (hi + lo, 8 k-steps) in registers and runs over its M tiles of 16 rows:
// A operands come from LDS (16 bytes per lane: row m, columns ks*32 + kq*8).
// ------------------------------------------------------------------------------------------------
constexpr int XL_RB = 128;               // rows per workgroup
constexpr int XL_KC = 128;               // columns per chunk
constexpr int XL_KS = XL_KC / 32;        // k-steps per chunk
constexpr int XL_PITCH = XL_KC + 8;      // bf16 elements per staged row (16 bytes of padding)
constexpr int XL_AHEAD = 4;              // chunks of X in flight from HBM (register sets)

template <int P>
__global__ __launch_bounds__(512) void xscores_kernel(const uint16_t* qt, const uint16_t* X, long x_bstride,
                                                      const int32_t* seq_lens, int T, int B, int H, int dm, float* S,
                                                      int colocate) {
  __shared__ __align__(16) uint16_t xs[2][XL_RB * XL_PITCH];
  constexpr int RS = 8 / P;                            // waves per head tile = row subsets
  constexpr int D = XL_AHEAD;
  // unit = sequence (its row blocks read the same q~), inner = block of XL_RB rows
  int b, rbk;
  if (!unit_of_workgroup(blockIdx.x, (T + XL_RB - 1) / XL_RB, B, colocate != 0, b, rbk)) return;
  const int row_base = rbk * XL_RB;
  const int len = seq_len_of(seq_lens, b, T);
  if (row_base >= len) return;                         // (workgroup-uniform)
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int n = lane & 15, kq = lane >> 4;
  const int htl = w % P, rs = w / P;
  const int NHT = (H + 15) / 16;
  const int nkc = dm / XL_KC, npass = (NHT + P - 1) / P;   // (dm is a multiple of 128)
  const int total = npass * nkc;
  const uint16_t* Xb = X + (size_t)b * x_bstride;
  const size_t lo_off = (size_t)B * NHT * 16 * dm;     // the lo halves follow the hi halves
  const int Tp = (T + 31) / 32 * 32;                   // rows of S are padded to whole tiles

  // staging: thread t moves 16-byte column chunk t % 16 of rows t / 16 + 32 i
  const int srow = tid >> 4, scol = (tid & 15) * 8;
  u32x4 stg[D][4];
  auto issue_x = [&](u32x4 (&g)[4], int it) {
    const int col = (it % nkc) * XL_KC + scol;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = min(row_base + srow + 32 * i, len - 1);   // rows past the end: any finite values, never stored
      g[i] = *reinterpret_cast<const u32x4*>(Xb + (size_t)r * dm + col);
    }
  };
  auto commit_x = [&](const u32x4 (&g)[4], int it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<u32x4*>(&xs[it & 1][(srow + 32 * i) * XL_PITCH + scol]) = g[i];
  };
  // B operands of iteration it (head tile and chunk): 1 KB of consecutive bytes per operand
  auto load_b = [&](u32x4 (&bh)[XL_KS], u32x4 (&bl)[XL_KS], int it) {
    const int ht = min((it / nkc) * P + htl, NHT - 1), kc = it % nkc;
    const uint16_t* src = qt + ((((size_t)b * NHT + ht) * (dm / 32) + (size_t)kc * XL_KS) * 64 + lane) * 8;
#pragma unroll
    for (int ks = 0; ks < XL_KS; ++ks) {
      bh[ks] = *reinterpret_cast<const u32x4*>(src + ks * 512);
      bl[ks] = *reinterpret_cast<const u32x4*>(src + lo_off + ks * 512);
    }
  };

  f32x4 acc[P];
  u32x4 bh[XL_KS], bl[XL_KS], nh[XL_KS], nl[XL_KS];
#pragma unroll
  for (int j = 0; j < D; ++j) issue_x(stg[j], min(j, total - 1));
  load_b(bh, bl, 0);
  commit_x(stg[0], 0);
  lds_barrier();
  // One chunk; SI is it % D as a type: the register set whose chunk (it) has already gone to LDS.
  auto step = [&](int it, auto SI) {
    constexpr int si = decltype(SI)::value;
    const int hp = it / nkc, kc = it % nkc;
    const bool more = it + 1 < total;
    // (a wave's loads complete in issue order: what the next chunk needs goes first, so that waiting for it
    //  does not wait for the X chunk that is D chunks away)
    // Issued unconditionally (past the end: the last chunk again, unused) so that the compiler can count
    // the loads in flight and wait for exactly the ones a step needs.
    load_b(nh, nl, min(it + 1, total - 1));
    issue_x(stg[si], min(it + D, total - 1));
    const int ht = hp * P + htl;
    if (kc == 0) {
#pragma unroll
      for (int mi = 0; mi < P; ++mi) acc[mi] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    if (ht < NHT) {
      const uint16_t* xa = &xs[it & 1][n * XL_PITCH + kq * 8];
#pragma unroll
      for (int mi = 0; mi < P; ++mi) {
        const int mt = rs + mi * RS;                   // this wave's M tiles: rs, rs + RS, ...
#pragma unroll
        for (int ks = 0; ks < XL_KS; ++ks) {
          const bf16x8 a8 = *reinterpret_cast<const bf16x8*>(xa + mt * 16 * XL_PITCH + ks * 32);
          acc[mi] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8, __builtin_bit_cast(bf16x8, bh[ks]), acc[mi], 0, 0, 0);
          acc[mi] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8, __builtin_bit_cast(bf16x8, bl[ks]), acc[mi], 0, 0, 0);
        }
      }
      if (kc == nkc - 1) {                             // D: column n = head, rows kq*4 + r
        const int h = ht * 16 + n;
        if (h < H) {
#pragma unroll
          for (int mi = 0; mi < P; ++mi) {
            const int t0 = row_base + (rs + mi * RS) * 16 + kq * 4;
            float* dst = S + ((size_t)b * H + h) * Tp + t0;
            if (t0 + 3 < len) {                         // (rows of S are padded to 32: 16-byte aligned)
              *reinterpret_cast<f32x4*>(dst) = acc[mi];
            } else {
#pragma unroll
              for (int r = 0; r < 4; ++r)
                if (t0 + r < len) dst[r] = acc[mi][r];
            }
          }
        }
      }
    }
    if (more) {
      commit_x(stg[(si + 1) % D], it + 1);
#pragma unroll
      for (int ks = 0; ks < XL_KS; ++ks) { bh[ks] = nh[ks]; bl[ks] = nl[ks]; }
    }
    lds_barrier();
  };
  int it = 0;
  for (; it + D <= total; it += D) full_steps<0, D>(it, step);
  unrolled_steps<0, D>(it, total, step);
}

// ------------------------------------------------------------------------------------------------
// Weighted sum of the rows of X for one (sequence, context split, group of 32 heads, block of 128
// columns).  The 8 waves of the workgroup split the ROWS of the split (wave w takes 32-row tiles w,
// w + 8, ...) and merge their (m, l, C) through LDS at the end, so one partial leaves per workgroup:
// splitting the context across workgroups instead costs H x d_model x 4 bytes of partial per split and
// sequence, which at 8 splits was four times the bytes of X itself.
// Register tile and MFMA layout as in the K-cache stream kernel: lane (idx = l % 16, rg = l / 16)
// loads 16 bytes of rows rg*8 .. rg*8+7, transposes its 8x8 block into 8 A operands; B = weights
// P^T (lane (n = head, kg = row group) reads 8 consecutive scores of head n).
// Writes Cpart[(b nsplit + s)][h][c] (unnormalised), mpart (log2 domain) and lpart.
// ------------------------------------------------------------------------------------------------
constexpr float XW_SLACK = 6.0f;

__global__ __launch_bounds__(512) void xweighted_kernel(const float* S, const uint16_t* X, long x_bstride,
                                                        const int32_t* seq_lens, int T, int B, int H, int dm, int nsplit,
                                                        float* Cpart, float* mpart, float* lpart, int colocate) {
  constexpr int NT = 2, NW = 8;
  __shared__ float red[NW][NT][4][8][64];              // [wave][head tile][r][i][lane]: 128 KB
  __shared__ float msh[NW][NT * 16], lsh[NW][NT * 16];
  // unit = (sequence, context split): its workgroups read the same rows of X (one column block each, for
  // every head group) and the same scores (one head group each, for every column block)
  const int ncb = dm / 128;
  int unit, inner;
  if (!unit_of_workgroup(blockIdx.x, ((H + 31) / 32) * ncb, B * nsplit, colocate != 0, unit, inner)) return;
  const int b = unit / nsplit, s = unit - b * nsplit;
  const int cbk = inner % ncb, hg = inner / ncb;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int idx = lane & 15, rg = lane >> 4;
  const int n = idx, kg = rg;
  const int col0 = cbk * 128;
  const int len = seq_len_of(seq_lens, b, T);
  const int rows_per = ((len + nsplit - 1) / nsplit + 31) / 32 * 32;
  const int r_lo = s * rows_per, r_hi = min(len, r_lo + rows_per);
  const int pid = b * nsplit + s;
  const int ntile_all = r_lo < r_hi ? (r_hi - r_lo + 31) / 32 : 0;
  const int ntile = ntile_all > w ? (ntile_all - w + NW - 1) / NW : 0;   // this wave's tiles: w, w + 8, ...
  auto row_of = [&](int k) { return r_lo + 32 * (w + NW * k); };

  float m[NT];
  f32x4 acc[8][NT], accl[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    m[t] = NEG_INF;
    accl[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i][t] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  // Rows are addressed by 32-bit byte offsets from the sequence's base (a sequence of X is below 4 GB:
  // checked on the host); rows past the end re-read the last row and weigh nothing (their scores are masked).
  const char* Xb = reinterpret_cast<const char*>(X + (size_t)b * x_bstride + col0 + idx * 8);
  const unsigned pitchB = (unsigned)dm * 2u;
  auto load_tile = [&](u32x4 (&t)[8], int r0) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const unsigned off = __umul24((unsigned)min(r0 + rg * 8 + j, len - 1), pitchB);
      t[j] = *reinterpret_cast<const u32x4*>(Xb + off);
    }
  };
  // scores of a tile: lane (n, kg) takes rows r0 + kg*8 .. +7 of heads hg*32 + t*16 + n.  The rows of S
  // are padded to a multiple of 32 floats, so the 32 bytes are always there; what lies past the end of
  // the split (or belongs to a padded head) is replaced, not computed with.
  const int Tp = (T + 31) / 32 * 32;
  auto load_scores = [&](f32x4 (&x)[NT][2], int r0) {    // (raw: masked when used, so that nothing waits here)
    const int row = r0 + kg * 8;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int h = min(hg * 32 + t * 16 + n, H - 1);
      const float* src = S + ((size_t)b * H + h) * Tp + row;
      x[t][0] = *reinterpret_cast<const f32x4*>(src);
      x[t][1] = *reinterpret_cast<const f32x4*>(src + 4);
    }
  };
  // X tiles travel HBM/L2 -> registers D tiles ahead, scores DS tiles ahead (register sets chosen by a
  // compile-time index).  A step's work is short next to the latency of a load, so what it needs must
  // have been requested several steps earlier.  Loads past the end re-read the last tile (unused) so that
  // every step issues the same loads and the compiler can wait for exactly the ones a step needs.
  constexpr int D = 2, DS = 2, UN = 2;                 // X sets, score sets, steps per unrolled group (a common multiple)
  u32x4 xt[D][8];
  f32x4 sc[DS][NT][2];
  if (ntile > 0) {
#pragma unroll
    for (int j = 0; j < DS; ++j) load_scores(sc[j], row_of(min(j, ntile - 1)));
#pragma unroll
    for (int j = 0; j < D; ++j) load_tile(xt[j], row_of(min(j, ntile - 1)));
  }
  auto step = [&](int k, auto SI) {
    constexpr int si = decltype(SI)::value;
    u32x4 (&cur)[8] = xt[si % D];
    f32x4 (&sx)[NT][2] = sc[si % DS];
    const int row = row_of(k) + kg * 8;
    bf16x8 pb[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int live = (hg * 32 + t * 16 + n < H) ? r_hi - row : 0;   // rows of this lane that count
      float x[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) x[j] = j < live ? sx[t][j >> 2][j & 3] : NEG_INF;
      float tmax = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
      // The reference the weights are taken against moves only when the maximum has grown by more than
      // XW_SLACK (log2 domain): weights stay below 2^XW_SLACK, which costs bf16 and the fp32 sums nothing,
      // and the accumulators are rescaled rarely instead of at nearly every tile.
      const float mn = (tmax > m[t] + XW_SLACK) ? tmax : m[t];
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
    // both sets are free again: the scores of the wave's tile k + DS first, then X of its tile k + D
    load_scores(sx, row_of(min(k + DS, ntile - 1)));
    load_tile(cur, row_of(min(k + D, ntile - 1)));
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
  };
  int k = 0;
  for (; k + UN <= ntile; k += UN) full_steps<0, UN>(k, step);
  unrolled_steps<0, UN>(k, ntile, step);

  // ---- merge the 8 waves: common maximum per head, rescale, sum through LDS ---------------------
  // (a lane's accumulators of head tile t all belong to head t*16 + n: the D operand's column)
  if (kg == 0) {
#pragma unroll
    for (int t = 0; t < NT; ++t) msh[w][t * 16 + n] = m[t];
  }
  __syncthreads();
  float mall[NT];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    float mm = NEG_INF;
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) mm = fmaxf(mm, msh[ww][t * 16 + n]);
    mall[t] = mm;
    const float sc = (m[t] == NEG_INF) ? 0.f : __builtin_amdgcn_exp2f(m[t] - mm);
    if (kg == 0) lsh[w][t * 16 + n] = accl[t][0] * sc;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) red[w][t][r][i][lane] = acc[i][t][r] * sc;
  }
  __syncthreads();
  // thread (t, r, lane): columns col0 + (rg*4 + r)*8 .. +7 of head hg*32 + t*16 + n
  {
    const int t = w >> 2, r = w & 3;
    const int h = hg * 32 + t * 16 + n;
    float o[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float sum = 0.f;
#pragma unroll
      for (int ww = 0; ww < NW; ++ww) sum += red[ww][t][r][i][lane];
      o[i] = sum;
    }
    if (h < H) {
      float* dst = Cpart + ((size_t)pid * H + h) * dm + col0 + (rg * 4 + r) * 8;
      *reinterpret_cast<f32x4*>(dst) = f32x4{o[0], o[1], o[2], o[3]};
      *reinterpret_cast<f32x4*>(dst + 4) = f32x4{o[4], o[5], o[6], o[7]};
      if (cbk == 0 && r == 0 && kg == 0) {
        float l = 0.f;
#pragma unroll
        for (int ww = 0; ww < NW; ++ww) l += lsh[ww][t * 16 + n];
        mpart[(size_t)pid * H + h] = mall[t];
        lpart[(size_t)pid * H + h] = l;
      }
    }
  }
}


// ------------------------------------------------------------------------------------------------
// One pass over X for 512 <= d_model <= 1280: scores, softmax numerators and the weighted sum of one
// (sequence, context split, group of heads) in one kernel, so X leaves memory once per head group,
// no score matrix is written, and the exponentials of a row are computed once instead of once per
// column block.  The accumulators (32 heads x d_model fp32 = 128 KB at 1024 columns) stay in the
// workgroup's registers for its whole row range, which is why the COLUMNS are split over the waves
// (wave w owns columns [128 w, 128 w + 128): its slice of q~ as resident B operands, its 32 x 128 slice
// of every row tile, its accumulator block) and the waves meet twice per 32-row tile in LDS --
// the same exchange of numerators between column owners as in the K-cache stream kernel, but inside
// one workgroup, with barriers:
//   1. park the slice in LDS (row-padded), transpose it in registers for step 3, request the next tile,
//      read the slice back in A-operand order, partial scores of the group's heads over the wave's
//      columns on MFMA (query hi + lo), partials to LDS;  -- barrier --
//   2. waves 0..7 sum the partials of their heads over the column owners (lane = row), keep those
//      heads' running reference and sum of weights, write bf16 numerators and the rescale factors;
//      -- barrier --
//   3. every wave rescales if a reference moved and adds P^T X on MFMA.
// Rows are not split over the waves, so nothing is merged at the end.  A one-dimensional launch: the head
// groups of a (sequence, context split) read the same rows and are mapped to one XCD (unit_of_workgroup).
// Two shapes: 8 waves x 32 heads (d_model <= 1024; 32 + 16 MFMAs per wave and tile) and 10 waves x 16
// heads (d_model <= 1280: three waves on two of the four SIMDs, hence 168 registers, which hold half
// the accumulators and the hi halves of q~; the lo halves wait in LDS).
// ------------------------------------------------------------------------------------------------
// max over the 32 lanes that share lane / 32: four DPP steps inside the 16-lane row (lane ^ 1, lane ^ 2,
// the other quad of the 8-lane half, the other half of the row), then the row 16 lanes away by a register swap
template <int CTRL>
__device__ __forceinline__ float dpp_max(float v) {
  return fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true)));
}
__device__ __forceinline__ float max_over_32(float v) {
  v = dpp_max<0xB1>(v);
  v = dpp_max<0x4E>(v);
  v = dpp_max<0x141>(v);
  v = dpp_max<0x140>(v);
  const unsigned u = __float_as_uint(v);
  const auto sw = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}

constexpr int XF_PITCH = 272;            // bytes per parked row: 256 + 16 of padding
constexpr int XF_RED_HS = 36;            // floats per head row of a wave's partial scores (32 rows + padding that keeps 16-byte stores)
constexpr int XF_P_HS = 40;              // bf16 per head row of the numerators (32 rows + padding)

// NW waves, each the owner of 128 columns (d_model <= 128 NW); NT head tiles of 16 per group.  Two shapes are
// built: 8 waves x 32 heads (two waves per SIMD, 256 registers each) and 10 waves x 16 heads for rows of up to
// 1280 columns (three waves on two of the SIMDs: 168 registers, which half the accumulators and half the
// resident q~ fit).  The softmax state of the group's heads is looked after by waves 0..7, HG / 8 heads each.
template <int NW, int NT>
__global__ __launch_bounds__(NW * 64) void xfused_kernel(const uint16_t* qt, const uint16_t* X, long x_bstride,
                                                         const int32_t* seq_lens, int T, int B, int H, int dm, int nsplit,
                                                         float* Cpart, float* mpart, float* lpart, int colocate) {
  constexpr int HG = 16 * NT;                          // heads per group
  constexpr int HPL = HG / 16;                         // heads per lane of an owner wave (lane = (row, half): 2 x 32 lanes)
  static_assert(NW >= 8 && (NT == 1 || NT == 2), "owners are waves 0..7");
  __shared__ __align__(16) unsigned char slot[NW][32 * XF_PITCH];
  __shared__ __align__(16) float red[NW][HG][XF_RED_HS];
  __shared__ __align__(16) uint16_t P_s[HG][XF_P_HS];
  __shared__ float alpha_s[HG];
  // With three waves per SIMD the lo halves of q~ do not fit the registers: they wait in LDS (a wave's own
  // 4 KB, read back one operand at a time); with two waves per SIMD they stay resident.
  constexpr bool LO_IN_LDS = NW > 8;
  __shared__ __align__(16) u32x4 qlo[LO_IN_LDS ? NW : 1][LO_IN_LDS ? NT * 4 : 1][64];
  // unit = (sequence, context split): its head groups read the same rows of X, from one XCD's L2
  int unit, hg;
  if (!unit_of_workgroup(blockIdx.x, (H + HG - 1) / HG, B * nsplit, colocate != 0, unit, hg)) return;
  const int b = unit / nsplit, s = unit - b * nsplit;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int idx = lane & 15, rg = lane >> 4;           // column group / row group of the register tile
  const int n = idx, kg = rg;                          // MFMA: N index (head) or M index (row), k group
  const int ncb = dm / 128;                            // column owners: waves 0 .. ncb - 1
  const bool has_cols = w < ncb;
  const int len = seq_len_of(seq_lens, b, T);
  const int rows_per = ((len + nsplit - 1) / nsplit + 31) / 32 * 32;
  const int r_lo = s * rows_per, r_hi = min(len, r_lo + rows_per);
  const int pid = b * nsplit + s;
  const int ntile = r_lo < r_hi ? (r_hi - r_lo + 31) / 32 : 0;
  const int NHT = (H + 15) / 16;

  // q~ of the group's 32 heads over this wave's columns, hi + lo, resident as B operands
  u32x4 bqh[NT][4], bql[LO_IN_LDS ? 1 : NT][4];
  {
    const size_t lo_off = (size_t)B * NHT * 16 * dm;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int ht = min(hg * NT + t, NHT - 1);        // (a tile past the last one repeats it; its heads are masked)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const uint16_t* src = qt + ((((size_t)b * NHT + ht) * (dm / 32) + (size_t)((has_cols ? w : 0) * 4 + ks)) * 64 + lane) * 8;
        bqh[t][ks] = *reinterpret_cast<const u32x4*>(src);
        if constexpr (LO_IN_LDS) qlo[w][t * 4 + ks][lane] = *reinterpret_cast<const u32x4*>(src + lo_off);
        else bql[t][ks] = *reinterpret_cast<const u32x4*>(src + lo_off);
      }
    }
  }
  const char* Xb = reinterpret_cast<const char*>(X + (size_t)b * x_bstride + (has_cols ? w * 128 : 0) + idx * 8);
  const unsigned pitchB = (unsigned)dm * 2u;
  // (rows past the end re-read the last row: finite values that meet a zero weight)
  auto load_tile = [&](u32x4 (&t)[8], int r0) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const unsigned off = __umul24((unsigned)max(min(r0 + rg * 8 + j, len - 1), 0), pitchB);
      t[j] = *reinterpret_cast<const u32x4*>(Xb + off);
    }
  };
  f32x4 acc[8][NT];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i][t] = f32x4{0.f, 0.f, 0.f, 0.f};
  // softmax state of the heads this wave owns (waves 0..7): lane (r = lane % 32, hp = lane / 32) looks after
  // row r of heads (2 w + hp) HPL + {0 .. HPL - 1} of the group; m is the same in all 32 lanes, l is the
  // lane's own share
  const int r = lane & 31, hp = lane >> 5;
  const bool owner = w < 8;
  float m[HPL], l[HPL];
#pragma unroll
  for (int i = 0; i < HPL; ++i) { m[i] = NEG_INF; l[i] = 0.f; }

  u32x4 xt[1][8];                                      // (one set: it is free again as soon as the tile is parked and transposed)
  auto tile_row = [&](int k) { return r_lo + 32 * min(k, max(ntile - 1, 0)); };
  load_tile(xt[0], tile_row(0));
  char* const sl = reinterpret_cast<char*>(slot[w]);

  u32x4 (&cur)[8] = xt[0];
  u32x4 am[8];                                         // the parked tile, transposed: A operands of its weighted sum
  // 1. the slice into LDS; partial scores of the 32 heads over this wave's 128 columns
  auto park = [&]() {
#pragma unroll
    for (int j = 0; j < 8; ++j) *reinterpret_cast<u32x4*>(sl + (rg * 8 + j) * XF_PITCH + idx * 16) = cur[j];
  };
  auto scores = [&](int k) {
    f32x4 sp[2][NT];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int t = 0; t < NT; ++t) sp[mt][t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const bf16x8 a8 = *reinterpret_cast<const bf16x8*>(sl + (mt * 16 + n) * XF_PITCH + (ks * 4 + kg) * 16);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          sp[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8, __builtin_bit_cast(bf16x8, bqh[t][ks]), sp[mt][t], 0, 0, 0);
          const u32x4 lo = LO_IN_LDS ? qlo[w][t * 4 + ks][lane] : bql[t][ks];
          sp[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8, __builtin_bit_cast(bf16x8, lo), sp[mt][t], 0, 0, 0);
        }
        // (three waves per SIMD: keep the scheduler from fetching all operands of the tile ahead, which
        //  would push the accumulators out of the registers)
        if constexpr (LO_IN_LDS) __builtin_amdgcn_sched_barrier(0);
      }
    if (has_cols) {                                    // D: column n = head, rows kg*4 + i
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int t = 0; t < NT; ++t) *reinterpret_cast<f32x4*>(&red[w][t * 16 + n][mt * 16 + kg * 4]) = sp[mt][t];
    }
  };
  // 2. this wave's four heads: sum over the column owners, reference, numerators
  auto numerators = [&](int k) {
    if (!owner) return;
    const int r0 = r_lo + 32 * k;
#pragma unroll
    for (int i = 0; i < HPL; ++i) {
      const int hl = (2 * w + hp) * HPL + i;
      float sc = 0.f;
#pragma unroll
      for (int w0 = 0; w0 < NW; w0 += 8) {             // (the reads of a batch are issued before the first is used)
        float part[8];
#pragma unroll
        for (int ws = 0; ws < 8; ++ws)                 // (waves without columns leave their block unwritten: read, not used)
          part[ws] = red[min(w0 + ws, NW - 1)][hl][r];
#pragma unroll
        for (int ws = 0; ws < 8; ++ws) sc += w0 + ws < ncb ? part[ws] : 0.f;
      }
      const bool live = (hg * HG + hl < H) && (r0 + r < r_hi);
      const float x = live ? sc : NEG_INF;
      const float tmax = max_over_32(x);
      // (the reference moves only when the maximum has grown by more than XW_SLACK, as in xweighted_kernel)
      const float mn = (tmax > m[i] + XW_SLACK) ? tmax : m[i];
      const float ref = (mn == NEG_INF) ? 0.f : mn;
      const float alpha = (m[i] == NEG_INF) ? 1.f : __builtin_amdgcn_exp2f(m[i] - ref);   // (nothing accumulated yet: nothing to rescale)
      const __bf16 pw = (__bf16)__builtin_amdgcn_exp2f(x - ref);
      l[i] = l[i] * alpha + (float)pw;                 // the weight as the MFMA will see it
      m[i] = mn;
      P_s[hl][r] = __builtin_bit_cast(uint16_t, pw);
      if (r == 0) alpha_s[hl] = alpha;
    }
  };
  // 3. rescale where a reference moved; P^T X for this wave's columns (the tile in am, its numerators in LDS)
  auto weighted_sum = [&]() {
    bf16x8 pb[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const float al = alpha_s[t * 16 + n];
      pb[t] = *reinterpret_cast<const bf16x8*>(&P_s[t * 16 + n][kg * 8]);
      if (__any(al != 1.f)) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i][t] *= al;
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bf16x8 av = __builtin_bit_cast(bf16x8, am[i]);
#pragma unroll
      for (int t = 0; t < NT; ++t) acc[i][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, pb[t], acc[i][t], 0, 0, 0);
    }
  };
  // (Letting the weighted sum of tile k - 1 share a barrier interval with the scores of tile k, the two waves
  //  of a SIMD in opposite order, was measured: 68 against 58 us on the T5-11B-shaped configuration.)
  for (int k = 0; k < ntile; ++k) {
    park();
    transpose8x8(cur, am);                             // (cur is parked: its registers go to the next tile,
    // requested before the scores so that it has a whole step to arrive; past the end: the last tile again,
    // unused)
    load_tile(cur, tile_row(k + 1));
    scores(k);
    lds_barrier();
    numerators(k);
    lds_barrier();
    weighted_sum();
  }

  // ---- the partial of this (sequence, split): every wave its own columns, the owners their heads' (m, l).
  // An accumulator lane holds 32 consecutive columns of one head as eight 16-byte pieces: stored from there,
  // every instruction writes 64 pieces into 64 different cache lines (measured: 10 of the kernel's 59 us on
  // 8 sequences x 128 heads x 1024 columns).  So the wave's 16 x 128 block of a head tile goes through its
  // own, now idle, slot and leaves with a head's 512 bytes on 32 consecutive lanes.
  if (has_cols) {
    constexpr int OP = 128 + 4;                        // floats per head row in the slot (padding: no bank conflicts)
    static_assert(16 * OP * 4 <= 32 * XF_PITCH, "a head tile's block must fit the wave's slot");
    float* const ob = reinterpret_cast<float*>(sl);
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // (the wave's earlier reads of the slot are done)
#pragma unroll
      for (int i = 0; i < 4; ++i) {                    // accumulator row i: column group rg*4 + i of the block
        float* d8 = ob + n * OP + (rg * 4 + i) * 8;
        *reinterpret_cast<f32x4*>(d8) = f32x4{acc[0][t][i], acc[1][t][i], acc[2][t][i], acc[3][t][i]};
        *reinterpret_cast<f32x4*>(d8 + 4) = f32x4{acc[4][t][i], acc[5][t][i], acc[6][t][i], acc[7][t][i]};
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // (LDS operations of one wave complete in order)
#pragma unroll
      for (int k2 = 0; k2 < 8; ++k2) {
        const int hl = 2 * k2 + (lane >> 5), c4 = (lane & 31) * 4;
        const int h = hg * HG + t * 16 + hl;
        const f32x4 v = *reinterpret_cast<const f32x4*>(ob + hl * OP + c4);
        if (h < H) *reinterpret_cast<f32x4*>(Cpart + ((size_t)pid * H + h) * dm + w * 128 + c4) = v;
      }
    }
  }
#pragma unroll
  for (int i = 0; i < HPL; ++i) {
    float lt = l[i];
#pragma unroll
    for (int o = 1; o < 32; o <<= 1) lt += __shfl_xor(lt, o);
    const int h = hg * HG + (2 * w + hp) * HPL + i;
    if (owner && r == 0 && h < H) {
      mpart[(size_t)pid * H + h] = m[i];
      lpart[(size_t)pid * H + h] = lt;
    }
  }
}

}  // namespace

// Head tiles in flight for H heads: 1, 2, 4 or 8.
static int head_tiles_in_flight(int H) {
  const int nht = (H + 15) / 16;
  int p = 1;
  while (p < nht && p < 8) p *= 2;
  return p;
}
bool xcache_fast_ok(int dtype, int H, int d_model, int d_k) {
  return dtype == DT_BF16 && d_model % 128 == 0 && d_k % 32 == 0 && d_k >= 32 && H >= 1 && d_model < (1 << 22);
}

int xcache_splits(int B, int H, int T, int d_model) {
  // The weighted sum runs one workgroup per (split, 32 heads, 128 columns, sequence): split the context
  // across workgroups only as far as it takes to fill the chip (every split costs a partial).
  const int per = B * ((H + 31) / 32) * (d_model >= 128 ? d_model / 128 : 1);
  int s = (256 + per - 1) / per;
  const int cap = (T + 255) / 256;
  if (s > cap) s = cap;
  if (s > PROJ_MAX_PARTS) s = PROJ_MAX_PARTS;
  return s < 1 ? 1 : s;
}

bool xfused_ok(int d_model) { return d_model % 128 == 0 && d_model >= 512 && d_model <= 1280; }

// heads per workgroup of the one-pass kernel: 32 with 8 column owners, 16 with 10 (rows wider than 1024)
static int xfused_head_group(int d_model) { return d_model <= 1024 ? 32 : 16; }

int xfused_splits(int B, int H, int T, int d_model) {
  // one workgroup per (split, head group, sequence): split the context as far as it takes to fill the chip
  const int hg = xfused_head_group(d_model);
  const int per = B * ((H + hg - 1) / hg);
  int s = (256 + per - 1) / per;
  const int cap = (T + 255) / 256;
  if (s > cap) s = cap;
  if (s > PROJ_MAX_PARTS) s = PROJ_MAX_PARTS;
  return s < 1 ? 1 : s;
}

// Units dealt to the 8 XCDs (unit_of_workgroup): only when they spread evenly, within a quarter
static int colocate_units(int nunits) { return (nunits % 8 == 0 || nunits >= 32) ? 1 : 0; }
static unsigned unit_grid(int nunits, int ninner, int colocate) {
  return colocate ? 8u * (unsigned)ninner * (unsigned)((nunits + 7) / 8) : (unsigned)nunits * (unsigned)ninner;
}

void launch_xfused(const float* qt, const void* X, long x_bstride, const int32_t* seq_lens, int T, int H, int d_model,
                   int nsplit, float* Cpart, float* mpart, float* lpart, int B, hipStream_t st) {
  const int hg = xfused_head_group(d_model);
  const int colocate = colocate_units(B * nsplit);
  dim3 grid(unit_grid(B * nsplit, (H + hg - 1) / hg, colocate));
  if (hg == 32)
    hipLaunchKernelGGL((xfused_kernel<8, 2>), grid, dim3(512), 0, st, (const uint16_t*)qt, (const uint16_t*)X, x_bstride, seq_lens, T, B, H,
                       d_model, nsplit, Cpart, mpart, lpart, colocate);
  else
    hipLaunchKernelGGL((xfused_kernel<10, 1>), grid, dim3(640), 0, st, (const uint16_t*)qt, (const uint16_t*)X, x_bstride, seq_lens, T, B, H,
                       d_model, nsplit, Cpart, mpart, lpart, colocate);
}

void launch_xq_tilde(const float* q, const void* Wk, float* qt, int B, int H, int d_k, int d_model, int e,
                     float scale, int* counters, int ncounters, hipStream_t st) {
  dim3 grid((H + XQ_HEADS - 1) / XQ_HEADS, (d_model + 127) / 128, (B + 15) / 16);
  hipLaunchKernelGGL(xq_tilde_kernel, grid, dim3(512), 0, st, q, (const uint16_t*)Wk, (uint16_t*)qt, B, H, d_k, d_model,
                     e, scale, counters, ncounters);
}

void launch_xscores(const float* qt, const void* X, long x_bstride, const int32_t* seq_lens, int T, int H,
                    int d_model, float* S, int B, hipStream_t st) {
  const int ninner = (T + XL_RB - 1) / XL_RB, colocate = colocate_units(B);
  dim3 grid(unit_grid(B, ninner, colocate));
  const uint16_t* q16 = (const uint16_t*)qt;
  const uint16_t* X16 = (const uint16_t*)X;
  switch (head_tiles_in_flight(H)) {
    case 1: hipLaunchKernelGGL(xscores_kernel<1>, grid, dim3(512), 0, st, q16, X16, x_bstride, seq_lens, T, B, H, d_model, S, colocate); break;
    case 2: hipLaunchKernelGGL(xscores_kernel<2>, grid, dim3(512), 0, st, q16, X16, x_bstride, seq_lens, T, B, H, d_model, S, colocate); break;
    case 4: hipLaunchKernelGGL(xscores_kernel<4>, grid, dim3(512), 0, st, q16, X16, x_bstride, seq_lens, T, B, H, d_model, S, colocate); break;
    default: hipLaunchKernelGGL(xscores_kernel<8>, grid, dim3(512), 0, st, q16, X16, x_bstride, seq_lens, T, B, H, d_model, S, colocate); break;
  }
}

void launch_xweighted(const float* S, const void* X, long x_bstride, const int32_t* seq_lens, int T, int H,
                      int d_model, int nsplit, float* Cpart, float* mpart, float* lpart, int B, hipStream_t st) {
  const int ninner = ((H + 31) / 32) * (d_model / 128), colocate = colocate_units(B * nsplit);
  dim3 grid(unit_grid(B * nsplit, ninner, colocate));
  hipLaunchKernelGGL(xweighted_kernel, grid, dim3(512), 0, st, S, (const uint16_t*)X, x_bstride, seq_lens, T, B, H,
                     d_model, nsplit, Cpart, mpart, lpart, colocate);
}

}  // namespace slim
