// bf16 fast path of the slim-attention decode step for gfx950 (MI355X).
//
//   fused_stream_kernel : one pass over the K-cache.  Softmax arguments (eq. 2), online softmax
//                         and the full-width weighted sum [softmax(.) K] of eq. 7 option 2, the
//                         latter as one MFMA contraction for all heads at once (the text under
//                         eq. 7 points out that the heads need not be handled one by one).  K is
//                         read from HBM once.
//   project_mfma_kernel : log-sum-exp merge of the context splits and the per-head product with
//                         W_KV,i (eq. 7 option 2, second factor) on MFMA; W_KV is read once.
//
// Why workgroups exchange scores.  The weighted sum keeps H x d fp32 accumulators per sequence
// (512 KB for H=32, d=4096: a whole CU's register file), so the row width has to be split over
// workgroups; but head h's weights need columns [h d_k, (h+1) d_k) only, which one column owner
// holds, while every column owner needs every head's weights.  A "group" of G workgroups (one per
// column unit of <=128 columns) therefore walks the same rows together; wave w of every workgroup of
// the group takes the same 32-row tiles: it computes the scores of the heads inside its unit, turns them
// into softmax numerators against the head's running reference, parks the tile in LDS and publishes
// 16-byte words {tag, reference, 4 bf16 numerators} to a small ring in global memory; one step later it
// gathers all heads' words of that tile, takes the tile out of LDS and feeds it to the MFMA.  No fences
// are needed: every 16-byte word (written by one store) carries the tile's tag, so a reader either
// sees the values of this tile or gathers again.  Every wait is bounded in real time; a time-out raises
// an error word instead of hanging.
//
// Register tile.  A wave owns 32 rows x 128 columns: lane l loads 16 bytes (8 columns) of 8 rows,
// column group l%16; the rows are 4 j + l/16 (one load instruction = four consecutive rows) or, with
// rotary keys, 8 (l/16) + j.  Both MFMA contractions take their operands from the tile's LDS
// copy.  Scores (v_mfma_f32_16x16x32_bf16, contraction over columns): A = 16 rows x 32 columns read
// straight in operand layout, B = the unit's queries.  Weighted sum (contraction over rows): a lane reads
// its 8 x 8 block back and transposes it in registers (v_perm_b32) into 8 A-operands, one per column:
// A_i[m = l%16][k = 8 rows of lane group l/16] = K[row][col (l%16)*8 + i]; the B-operand is P^T: lane
// (n = l%16, l/16) holds the weights of head n for the same 8 rows.
#include "slim_kernels.h"
#include "device_common.h"

#include <math.h>
#include <type_traits>

namespace slim {
namespace {

constexpr float LOG2E = 1.4426950408889634f;

__device__ __forceinline__ float bf16_lo(unsigned x) { return __uint_as_float(x << 16); }
__device__ __forceinline__ float bf16_hi(unsigned x) { return __uint_as_float(x & 0xffff0000u); }

// v + (v of the lane selected by a DPP control inside the 16-lane row); one v_add_f32_dpp
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
  return v + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// max over the four lanes l, l^16, l^32, l^48 (the same column group in the four row groups).
// Register swaps (v_permlane32_swap / v_permlane16_swap), no LDS traffic.
__device__ __forceinline__ float max_over_row_groups(float v) {
  const unsigned u = __float_as_uint(v);
  const auto a = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const float h = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  const unsigned w = __float_as_uint(h);
  const auto b = __builtin_amdgcn_permlane16_swap(w, w, false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

// Score exchange accesses.  Readers load at agent scope (never served by the CU's own vector L1).
// Writers have two flavours, chosen per launch:
//  * XCD-local (the normal case): all workgroups of a group run on one XCD (workgroup i is
//    dispatched to XCD i % 8, which the host verifies once per device), so that XCD's L2 is their
//    meeting point: a plain store (the vector L1 is write-through) is enough and the words never
//    leave the L2.
//  * system scope (fallback): write-through stores that also reach the memory side, for groups
//    whose workgroups may sit on different XCDs.
// 16-byte accesses: a wave's gather of one tile is a handful of fully coalesced 1 KB loads.
__device__ __forceinline__ u32x4 ld_exch(const u32x4* p) {
  u32x4 v;
  asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(p) : "memory");
  return v;
}
__device__ __forceinline__ void st_exch(u32x4* p, u32x4 v, bool xcd_local) {
  // The s_nops matter: a store of more than 64 bits still reads its data registers in the wait
  // states after it issues, and the compiler (which pads its own stores) is free to overwrite
  // the inputs of an asm statement with the very next VALU instruction.
  if (xcd_local) asm volatile("s_nop 1\n\tglobal_store_dwordx4 %0, %1, off\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
  else asm volatile("s_nop 1\n\tglobal_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
}
// Results other workgroups of the same launch will read (write_through): stored at system scope.
__device__ __forceinline__ void st_result(float* p, float v, bool write_through) {
  if (write_through) asm volatile("global_store_dword %0, %1, off sc0 sc1" : : "v"(p), "v"(v) : "memory");
  else *p = v;
}
__device__ __forceinline__ void st_result(int* p, int v, bool write_through) {
  if (write_through) asm volatile("global_store_dword %0, %1, off sc0 sc1" : : "v"(p), "v"(v) : "memory");
  else *p = v;
}

__device__ __forceinline__ void st_result4(float* p, f32x4 v, bool write_through) {
  // (s_nops: see st_exch)
  if (write_through) asm volatile("s_nop 1\n\tglobal_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" : : "v"(p), "v"(v) : "memory");
  else *reinterpret_cast<f32x4*>(p) = v;
}

// Tiles of 32 rows: prefix[b] = number of tiles of sequences 0..b-1; lens_s[b] (if given) = rows of
// sequence b.  The first wave takes 64 sequences at a time, one per lane (one memory round trip per 64
// sequences instead of one per sequence), and adds them up with a scan over the lanes.
__device__ void build_tile_prefix(int* prefix, int* lens_s, const int32_t* lens, int B, int T) {
  if (threadIdx.x < 64) {
    const int lane = threadIdx.x;
    int carry = 0;
    for (int b0 = 0; b0 < B; b0 += 64) {
      const int b = b0 + lane;
      const int len = b < B ? seq_len_of(lens, b, T) : 0;
      int v = (len + TILE_ROWS - 1) / TILE_ROWS;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(v, o);
        v += (lane >= o) ? up : 0;
      }
      if (b < B) {
        prefix[b + 1] = carry + v;
        if (lens_s) lens_s[b] = len;
      }
      carry += __shfl(v, 63);
    }
    if (lane == 0) prefix[0] = 0;
  }
  __syncthreads();
}

// ------------------------------------------------------------------------------------------------
// merge + projection:  out[b][h d_k + j] = sum_c Cn[b][h][c] W[c][h d_k + j]
// One workgroup (8 waves) per (head h, row split cs of W, batch chunk bz of 16*NBT sequences).  The
// wave tile is the same 32 x 128 register tile as above (rows = c, columns = the head's output
// columns), A = W tile transposed, B = merged, normalised C^T split in bf16 hi + lo.
// COH: the partials come from other workgroups of the same launch (loads at agent scope).
// ------------------------------------------------------------------------------------------------
template <int NBT>
struct ProjShared {
  int pid0s[16 * NBT], nps[16 * NBT];
  float wpid[16 * NBT][PROJ_MAX_PARTS];
  float obuf[16 * NBT][128];
  int is_last;
};

template <bool COH>
__device__ __forceinline__ float ld_part(const float* p) {
  if constexpr (COH) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else return *p;
}
template <bool COH>
__device__ __forceinline__ int ld_err(const int* p) {
  if constexpr (COH) return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  else return *p;
}

// `red`: 64 KB of LDS for the cross-wave sum.
// `after_w_issue` runs (all threads) once the first tile of W is in flight and before any partial
// is read: the place to build the tile prefix, or to wait for the other workgroups' partials.
// DENSE: plain products out_m = x W_m for up to three matrices that share x (ProjArgs::Wm); hx counts
// (matrix, head) column blocks.  The result leaves as fp32, or -- the new token's rows -- rotated to
// the append position and/or stored into the caches (ProjArgs::role).
template <int NBT, bool COH, bool DENSE, class Hook>
__device__ __forceinline__ void project_work(const ProjArgs& a, int hx, int cs, int bz, const int* prefix,
                                             ProjShared<NBT>& sm, float* red, Hook&& after_w_issue) {
  const int mtx = DENSE ? hx / a.H : 0;
  const int h = DENSE ? hx - mtx * a.H : hx;
  const uint16_t* const Wmat = DENSE ? a.Wm[mtx] : a.W;
  float* const outp = DENSE ? a.outm[mtx] : a.out;
  float* const outpart = DENSE ? a.outpart + (size_t)mtx * a.csw * a.B * a.e : a.outpart;
  const int bbase = bz * 16 * NBT;
  const int nb = min(16 * NBT, a.B - bbase);
  constexpr int NW = 8, NTHR = 512;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int idx = lane & 15, rg = lane >> 4;
  const int n = idx, kg = rg;

  const int nhx = DENSE ? a.H * a.nmat : a.H;          // arrival counters per batch chunk
  const int lph = a.d_k / 8;
  const bool col_active = idx < lph;
  // partial p of head h starts at ((p * H) + h) * rows; DENSE has one row of x per sequence for all heads
  const int hmul = DENSE ? 1 : a.H, hadd = DENSE ? 0 : h;
  const uint16_t* Wh = Wmat + (size_t)h * a.d_k + idx * 8;
  const int c_lo = cs * a.crows, c_hi = min(a.rows, c_lo + a.crows);
  const int ntile = (c_hi - c_lo + TILE_ROWS - 1) / TILE_ROWS;
  auto load_w = [&](u32x4 (&wt)[8], int ct) {
    const int c0 = c_lo + ct * TILE_ROWS;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int r = min(c0 + rg * 8 + j, a.rows - 1);
      wt[j] = col_active ? *reinterpret_cast<const u32x4*>(Wh + (size_t)r * a.e) : u32x4{0u, 0u, 0u, 0u};
    }
  };
  // DENSE: the B operand is a slice of x, known from the start: requested first, one tile ahead.
  f32x4 xc[NBT][2], xn[NBT][2];
  auto load_x = [&](f32x4 (&x)[NBT][2], int ct) {
    const int c = min(c_lo + ct * TILE_ROWS + kg * 8, a.rows - 8);
#pragma unroll
    for (int t = 0; t < NBT; ++t) {
      const float* src = a.Cpart + (size_t)min(bbase + t * 16 + n, a.B - 1) * a.rows + c;
      x[t][0] = *reinterpret_cast<const f32x4*>(src);
      x[t][1] = *reinterpret_cast<const f32x4*>(src + 4);
    }
  };
  if constexpr (DENSE) load_x(xc, min(w, max(ntile - 1, 0)));
  u32x4 wt[8], wn[8];
  if (w < ntile) load_w(wt, w);                      // in flight while the merge weights are built
  if (w + NW < ntile) load_w(wn, w + NW);

  after_w_issue();

  // ---- which partials belong to which sequence, and their merge weights for head h ------------
  for (int bl = w; bl < nb; bl += NW) {              // one wave per sequence, one lane per partial
    const int b = bbase + bl;
    int p0, np;
    if constexpr (DENSE) {                           // "partial" b is row b of x, weight 1
      if (lane == 0) { sm.wpid[bl][0] = 1.f; sm.pid0s[bl] = b; sm.nps[bl] = 1; }
      continue;
    }
    if (a.mode == 0) {
      const int VT = prefix[a.B];
      const int Qt = (VT + a.NG - 1) / a.NG;
      const int gf = prefix[b] / Qt, gl = (prefix[b + 1] - 1) / Qt;
      p0 = b + gf;
      np = gl - gf + 1;
    } else {
      p0 = b * a.nsplit;
      np = a.nsplit;
    }
    np = min(np, PROJ_MAX_PARTS);
    float mp = NEG_INF, lp = 0.f;
    if (lane < np) {
      mp = ld_part<COH>(a.mpart + (size_t)(p0 + lane) * a.H + h);
      lp = ld_part<COH>(a.lpart + (size_t)(p0 + lane) * a.H + h);
    }
    float M = mp;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) M = fmaxf(M, __shfl_xor(M, o));
    const float wgt = (mp == NEG_INF) ? 0.f : exp2f((mp - M) * a.mscale);
    float L = wgt * lp;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) L += __shfl_xor(L, o);
    if (lane < np) sm.wpid[bl][lane] = wgt / L;
    if (lane == 0) { sm.pid0s[bl] = p0; sm.nps[bl] = np; }
  }
  // (a barrier for the weights in LDS only: __syncthreads() would also wait for the tiles of W in flight)
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");

  f32x4 acc[8][NBT];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int t = 0; t < NBT; ++t) acc[i][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int ct = w; ct < ntile; ct += NW) {
    const int c0 = c_lo + ct * TILE_ROWS;
    const bool more = ct + NW < ntile;
    // B operand: merged C for (b = bt*16 + n, rows c0 + kg*8 .. +8)
    bf16x8 bhi[NBT], blo[NBT];
    const int c = c0 + kg * 8;
    if constexpr (DENSE) load_x(xn, min(ct + NW, ntile - 1));
#pragma unroll
    for (int t = 0; t < NBT; ++t) {
      float cn[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) cn[j] = 0.f;
      const int bl = t * 16 + n;
      if constexpr (DENSE) {
        if (bl < nb && c < c_hi) {
#pragma unroll
          for (int j = 0; j < 4; ++j) { cn[j] = xc[t][0][j]; cn[4 + j] = xc[t][1][j]; }
        }
      } else if (bl < nb && c < c_hi) {
        const int p0 = sm.pid0s[bl], np = sm.nps[bl];
        if constexpr (COH) {
          // eight partials per round trip: agent-scope loads, one wait
          for (int pb = 0; pb < np; pb += 8) {
            f32x4 x[8][2];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
              const int pp = min(pb + q, np - 1);
              const float* src = a.Cpart + ((size_t)(p0 + pp) * hmul + hadd) * a.rows + c;
              asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(x[q][0]) : "v"(src) : "memory");
              asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(x[q][1]) : "v"(src + 4) : "memory");
            }
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(x[0][0]), "+v"(x[0][1]), "+v"(x[1][0]), "+v"(x[1][1]),
                         "+v"(x[2][0]), "+v"(x[2][1]), "+v"(x[3][0]), "+v"(x[3][1]) : : "memory");
            asm volatile("" : "+v"(x[4][0]), "+v"(x[4][1]), "+v"(x[5][0]), "+v"(x[5][1]),
                         "+v"(x[6][0]), "+v"(x[6][1]), "+v"(x[7][0]), "+v"(x[7][1]) : : "memory");
#pragma unroll
            for (int q = 0; q < 8; ++q) {
              const float wgt = (pb + q < np) ? sm.wpid[bl][min(pb + q, np - 1)] : 0.f;
#pragma unroll
              for (int j = 0; j < 4; ++j) {
                cn[j] = fmaf(wgt, x[q][0][j], cn[j]);
                cn[4 + j] = fmaf(wgt, x[q][1][j], cn[4 + j]);
              }
            }
          }
        } else {
          for (int p = 0; p < np; ++p) {
            const float wgt = sm.wpid[bl][p];
            const float* src = a.Cpart + ((size_t)(p0 + p) * hmul + hadd) * a.rows + c;
            const float4 x0 = *reinterpret_cast<const float4*>(src);
            const float4 x1 = *reinterpret_cast<const float4*>(src + 4);
            cn[0] = fmaf(wgt, x0.x, cn[0]); cn[1] = fmaf(wgt, x0.y, cn[1]);
            cn[2] = fmaf(wgt, x0.z, cn[2]); cn[3] = fmaf(wgt, x0.w, cn[3]);
            cn[4] = fmaf(wgt, x1.x, cn[4]); cn[5] = fmaf(wgt, x1.y, cn[5]);
            cn[6] = fmaf(wgt, x1.z, cn[6]); cn[7] = fmaf(wgt, x1.w, cn[7]);
          }
        }
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const __bf16 hi = (__bf16)cn[j];
        bhi[t][j] = hi;
        blo[t][j] = (__bf16)(cn[j] - (float)hi);
      }
    }
    u32x4 am[8];
    transpose8x8(wt, am);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const bf16x8 av = __builtin_bit_cast(bf16x8, am[i]);
#pragma unroll
      for (int t = 0; t < NBT; ++t) {
        acc[i][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bhi[t], acc[i][t], 0, 0, 0);
        acc[i][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, blo[t], acc[i][t], 0, 0, 0);
      }
    }
    if (more) {
#pragma unroll
      for (int j = 0; j < 8; ++j) wt[j] = wn[j];
      if (ct + 2 * NW < ntile) load_w(wn, ct + 2 * NW);
    }
    if constexpr (DENSE) {
#pragma unroll
      for (int t = 0; t < NBT; ++t) { xc[t][0] = xn[t][0]; xc[t][1] = xn[t][1]; }
    }
  }

  // ---- sum the 8 waves: sm.obuf[b][j], IPR of the 8 accumulator columns per pass through LDS -----
  constexpr int IPR = 8 / NBT;
#pragma unroll
  for (int i0 = 0; i0 < 8; i0 += IPR) {
#pragma unroll
    for (int ii = 0; ii < IPR; ++ii)
#pragma unroll
      for (int t = 0; t < NBT; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[((w * IPR + ii) * (NBT * 4) + t * 4 + r) * 64 + lane] = acc[i0 + ii][t][r];
    __syncthreads();
    for (int v = tid; v < IPR * NBT * 4 * 64; v += NTHR) {
      const int ln = v & 63, reg = (v >> 6) % (NBT * 4), ii = (v >> 6) / (NBT * 4);
      float sum = 0.f;
#pragma unroll
      for (int ww = 0; ww < NW; ++ww) sum += red[((ww * IPR + ii) * (NBT * 4) + reg) * 64 + ln];
      const int t = reg >> 2, r = reg & 3;
      const int bl = t * 16 + (ln & 15);
      const int mi = (ln >> 4) * 4 + r;
      if (mi < lph) sm.obuf[bl][mi * 8 + i0 + ii] = sum;
    }
    __syncthreads();
  }

  // One finished output element (sequence bbase + bl, column j of the head); `other` is column j ^ 1.
  auto emit = [&](int bl, int j, float val, float other, bool bad) {
    const size_t b = (size_t)(bbase + bl);
    const int col = h * a.d_k + j;
    if constexpr (!DENSE) {
      outp[b * a.e + col] = bad ? NAN : val;
    } else {
      const int role = a.role[mtx];
      if (role == 0) { outp[b * a.e + col] = val; return; }
      // the new token of sequence b sits at row / position len_b - 1
      const int pos = seq_len_of(a.seq_lens, (int)b, a.T) - 1;
      if (pos < 0) return;
      float r = val;
      if (a.rope && (role == 1 || (role == 2 && a.rotate_k))) {
        const float* cs = a.rope + ((size_t)pos * (a.d_k / 2) + j / 2) * 2;
        r = (j & 1) ? fmaf(val, cs[0], -other * cs[1]) : fmaf(val, cs[0], other * cs[1]);
      }
      if (role == 1) { outp[b * a.e + col] = r; return; }
      // (banded K-cache: bands of 32 rows, a head's 32 x d_k block contiguous inside its band)
      const size_t at = (role == 2 && a.k_banded)
                            ? ((size_t)(pos >> 5) * a.H + h) * (32 * (size_t)a.d_k) + (size_t)(pos & 31) * a.d_k + j
                            : (size_t)pos * a.e + col;
      uint16_t* dst = (role == 2 ? a.Kc : a.Vc) + b * a.c_bstride + at;
      *dst = __builtin_bit_cast(uint16_t, (__bf16)r);
    }
  };

  if (a.csw == 1) {
    const bool bad = a.err && ld_err<COH>(a.err) == (int)a.launch_id;      // the stream kernel gave up waiting
    for (int v = tid; v < nb * a.d_k; v += NTHR) {
      const int bl = v / a.d_k, j = v % a.d_k;
      emit(bl, j, sm.obuf[bl][j], sm.obuf[bl][j ^ 1], bad);
    }
    return;
  }
  // ---- several workgroups share the rows of W: last one to arrive adds the partial sums ---------
  // No cache-wide fences: the partial sums are stored write-through and waited for (so they are
  // visible device-wide) before this workgroup's arrival is counted, and the last workgroup reads
  // them with device-coherent loads.
  for (int v = tid; v < nb * a.d_k; v += NTHR) {
    const int bl = v / a.d_k, j = v % a.d_k;
    float* dst = &outpart[((size_t)cs * a.B + bbase + bl) * a.e + h * a.d_k + j];
    asm volatile("global_store_dword %0, %1, off sc0 sc1" : : "v"(dst), "v"(sm.obuf[bl][j]) : "memory");
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (tid == 0) {
    const int old = __hip_atomic_fetch_add(&a.counters[bz * nhx + hx], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    sm.is_last = (old == a.csw - 1);
  }
  __syncthreads();
  if (!sm.is_last) return;
  // (the error word travels with the partial sums: requested here, looked at behind their wait)
  const int errv = a.err ? __hip_atomic_load(a.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
  for (int v0 = 0; v0 < nb * a.d_k; v0 += NTHR) {
    if (v0 + (tid & ~63) >= nb * a.d_k) break;           // (whole waves: the columns of a pair sit in neighbour lanes)
    const int v = min(v0 + tid, nb * a.d_k - 1);
    const int bl = v / a.d_k, j = v % a.d_k;
    float sum = 0.f;
    for (int s0 = 0; s0 < a.csw; s0 += 8) {
      float part[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int sp = min(s0 + q, a.csw - 1);
        const float* src = &outpart[((size_t)sp * a.B + bbase + bl) * a.e + h * a.d_k + j];
        asm volatile("global_load_dword %0, %1, off sc1" : "=v"(part[q]) : "v"(src) : "memory");
      }
      asm volatile("s_waitcnt vmcnt(0)" : "+v"(part[0]), "+v"(part[1]), "+v"(part[2]), "+v"(part[3]),
                   "+v"(part[4]), "+v"(part[5]), "+v"(part[6]), "+v"(part[7]) : : "memory");
#pragma unroll
      for (int q = 0; q < 8; ++q) if (s0 + q < a.csw) sum += part[q];
    }
    const float other = DENSE ? __shfl_xor(sum, 1) : 0.f;
    const bool bad = a.err && errv == (int)a.launch_id;
    if (v0 + tid < nb * a.d_k) emit(bl, j, sum, other, bad);               // NaN: the stream kernel gave up waiting
  }
  if (tid == 0) a.counters[bz * nhx + hx] = 0;
}

template <int NBT, bool DENSE>
__global__ __launch_bounds__(512) void project_mfma_kernel(const ProjArgs a) {
  __shared__ int prefix[FUSED_MAX_B + 1];
  __shared__ ProjShared<NBT> sm;
  __shared__ float red[8 * 8 * 4 * 64];
  project_work<NBT, false, DENSE>(a, blockIdx.x, blockIdx.y, blockIdx.z, prefix, sm, red, [&]() {
    if (!DENSE && a.mode == 0) build_tile_prefix(prefix, nullptr, a.seq_lens, a.B, a.T);
  });
}

// ------------------------------------------------------------------------------------------------
// fused stream kernel
//
// A workgroup is FUSED_WAVES waves that all do the same work on tiles of their own.  In step k a wave
//   1. parks tile k (in registers since two steps ago) in one of its two LDS slots and scores it from
//      there on MFMA (with rotary keys: on the vector ALU from the registers, before parking): scores of
//      its unit's heads, softmax numerators against the head's running maximum (bf16, the precision the
//      MFMA consumes anyway); publishes {tag, running max, 4 numerators} words,
//   2. requests all heads' words of its tile k-1 (published by the same wave of every workgroup of the
//      group one step earlier) and, behind them, tile k+2 into the registers that became free in 1,
//   3. takes tile k-1 out of its LDS slot while the words travel, waits for them (a wave's vector-memory
//      operations complete in issue order: the wait lets exactly the loads of tile k+2 stay in flight),
//      rescales its accumulators when a maximum moved and does the MFMA contraction.
// Every wave does both halves, so all eight waves of a compute unit share the scoring work and the
// loads.  A wave never waits for another wave of its workgroup.
// ------------------------------------------------------------------------------------------------
//
// ROPE (RoPE appendix, option 1): the cache holds raw keys and row t sits at position t.  The
// scoring rotates each key pair by its position for the score only; the tile that goes to the
// weighted sum stays raw.  With (y1, y2) = (x1 c + x2 s, -x1 s + x2 c) the pair's share of the
// score is c (q1 x1 + q2 x2) + s (q1 x2 - q2 x1): two dot products of the raw pair, with (q1, q2)
// and with (-q2, q1).  cos / sin of a lane's first row come from the table with the tile; the
// following seven rows advance by the one-position rotation (table row 1), kept in registers.
constexpr float SOFTMAX_SLACK = 6.0f;

// LPHP: lanes reserved per head as a compile-time constant (16 or 8: heads of 128 or 64 columns), or 0
// for the run-time value.  BYSEQ: the by-sequence partition (a.by_sequence != 0), which has no merge of the
// waves and never runs the projection; an instantiation of its own keeps each partition's code out of the
// other's registers.
template <int NT, bool ROPE, int LPHP, bool BYSEQ>
__global__ __launch_bounds__(FUSED_WAVES * 64) void fused_stream_kernel(const FusedArgs a) {
  constexpr int NP = FUSED_WAVES, NS = FUSED_SLOTS, PD = FUSED_AHEAD;
  constexpr int NTHR = NP * 64;
  constexpr int HP = NT * 16;                       // heads padded to the MFMA N tile
  static_assert(NP == 8 && NS == 2 && PD == 2, "the step structure and the thread mappings below assume these");
  __shared__ int prefix[FUSED_MAX_B + 1];
  __shared__ int lens_s[FUSED_MAX_B];               // rows per sequence
  __shared__ float marr[NP][NT][16];
  __shared__ float larr[NP][NT][16];
  // Per wave: NS landing slots of 8 KB for K tiles.  By-context partition: the end-of-share merge of
  // the waves goes through the (then idle) slots, which is why the array is a little larger than
  // the slots.  By-sequence partition: the other waves keep streaming; a wave writes its result
  // straight from its registers.  The projection of the single-launch mode runs after everything
  // else and reuses the slots and sbuf.
  constexpr int MERGE_PITCH = 132;                  // floats per head row of the merge buffer: 16-byte accesses without bank conflicts
  constexpr size_t SLOT_BYTES = (size_t)NP * NS * TILE_ROWS * 272, MERGE_BYTES = sizeof(float) * NP * HP * MERGE_PITCH;   // (272: a tile row and its padding)
  __shared__ __align__(16) unsigned char lds_main[SLOT_BYTES > MERGE_BYTES ? SLOT_BYTES : MERGE_BYTES];
  __shared__ __align__(16) float sbuf[sizeof(ProjShared<1>) / sizeof(float)];
  float* const mbuf = reinterpret_cast<float*>(lds_main);           // [NP][HP][MERGE_PITCH] floats
  float* const red = reinterpret_cast<float*>(lds_main);            // 64 KB for the projection's cross-wave sum
  static_assert(sizeof(float) * 8 * 8 * 4 * 64 <= sizeof(lds_main), "cross-wave sum must fit");

  // ---- which group / column unit is this workgroup -------------------------------------------
  int g = 0, u = 0;
  bool has_work = true;                             // (workgroup-uniform)
  {
    const int i = blockIdx.x;
    if (a.gpx > 0) {                                // groups packed inside one XCD (WG i -> XCD i % 8)
      const int x = i & 7, r = i >> 3;
      const int gx = r / a.G;
      if (gx >= a.gpx) has_work = false;
      g = x * a.gpx + gx;
      u = r % a.G;
    } else {
      g = i / a.G;
      u = i % a.G;
    }
    if (g >= a.NG) has_work = false;
  }
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int idx = lane & 15, rg = lane >> 4;        // column group / row group of the register tile
  const int n = idx, kg = rg;                       // head-in-tile / row group of the B operand
  const int wu = __builtin_amdgcn_readfirstlane(w);
  const int p = wu;                                 // this wave's team: wave p of every workgroup of the group

  const bool fuse = !BYSEQ && a.fuse != 0;
  if (blockIdx.x == 0 && a.counters)                // the projection's arrival counters start at 0
    for (int i = tid; i < a.ncounters; i += NTHR) st_result(a.counters + i, 0, fuse);

  build_tile_prefix(prefix, lens_s, a.seq_lens, a.B, a.T);     // (ends with a workgroup barrier)
  const int VT = prefix[a.B];
  const int Qt = (VT + a.NG - 1) / a.NG;            // tiles per group
  const int v0 = g * Qt, v1 = min(VT, v0 + Qt);
  if (BYSEQ ? (g * NP >= a.B * a.by_sequence) : (v0 >= v1)) has_work = false;
  if (!has_work && !fuse) return;

  // ---- lane -> column mapping inside the unit --------------------------------------------------
  const int lphp = LPHP ? LPHP : a.lphp;
  const int hh = idx / lphp, li = idx % lphp;
  const int myhead = u * a.hpu + hh;
  const bool col_active = (li < a.lph) && (hh < a.hpu) && (myhead < a.H);
  const int mycol = myhead * a.d_k + li * 8;        // first of this lane's 8 columns
  const bool pub_lane = col_active && (li == 0);    // one lane per head publishes its row group
  const int ucol0 = u * a.hpu * a.d_k;
  const int uwc = min(a.hpu * a.d_k, a.d - ucol0);  // columns of this unit
  int ocol[4];                                      // first unit-local column of accumulator row r, or -1
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int mi = rg * 4 + r;                      // column group (the A operand's M index)
    const int h2 = mi / lphp, l2 = mi % lphp;
    ocol[r] = (l2 < a.lph && h2 < a.hpu && h2 * a.d_k + l2 * 8 < uwc) ? h2 * a.d_k + l2 * 8 : -1;
  }

  // A tile in its LDS slot: row r, 16-byte chunk c (8 columns) at byte r * ROW_PITCH + c * 16, with one
  // chunk of padding per row (17 chunks), so that all three access patterns are free of bank conflicts
  // and each is one per-lane base plus compile-time offsets: the store and the read for the weighted sum
  // (the 16 chunks of a row) and the A operands of the score MFMA (one chunk of 16 consecutive rows).
  //   store of register j (row j*RJ + rg*RR), chunk idx ....... wpos + j * RJ * ROW_PITCH
  //   score A operand, rows mt*16 + idx, chunk ks*4 + rg ...... spos + mt * 16 * ROW_PITCH + ks * 64
  //   sum, rows jh*16 + kg*4 + jl, chunk idx (no rotary keys) . ppos + (jh * 16 + jl) * ROW_PITCH
  constexpr unsigned ROW_PITCH = 272, SLOT_PITCH = TILE_ROWS * ROW_PITCH;
  // Which row of the tile a lane's register j holds: j * RJ + rg * RR.  With rotary keys the scores are taken
  // from the registers and a lane needs eight consecutive positions (rows rg*8 + j).  Otherwise the registers
  // only carry the tile to its slot, and row j*4 + rg makes one load instruction cover four consecutive rows:
  // in the banded cache 4 d_k x 2 contiguous bytes, whole cache lines that no other instruction touches
  // (with rows eight apart and d_k = 96, every second line is shared by two instructions).
  constexpr int RJ = ROPE ? 1 : 4, RR = ROPE ? 8 : 1;
  const unsigned wpos = (unsigned)(rg * RR) * ROW_PITCH + (unsigned)idx * 16u;
  const unsigned spos = (unsigned)idx * ROW_PITCH + (unsigned)rg * 16u;
  const unsigned ppos = (unsigned)(kg * 4) * ROW_PITCH + (unsigned)idx * 16u;
  // Scores on MFMA (no rotary keys): column n = 2 * (head in unit) + {0: query hi, 1: query lo}; the lane
  // with the even n publishes its head's words for its four-row groups.
  const int mhead = u * a.hpu + (idx >> 1);          // head of this lane's score column
  const bool mpub_lane = !(idx & 1) && (idx >> 1) < a.hpu && mhead < a.H;

  const bool xl = a.xcd_local != 0;
  const bool heads_full = (a.H == HP);               // no padded heads in the MFMA N tiles
  const unsigned pitchB = (unsigned)a.d * 2u;        // bytes per cache row
  u32x4* const team_ring = reinterpret_cast<u32x4*>(a.exch) + (size_t)(g * NP + p) * EXCH_SLOTS * (HP * 8);
  char* const myslots = reinterpret_cast<char*>(lds_main) + (size_t)p * NS * SLOT_PITCH;
  bool dead = false;                                // a wait timed out: stop waiting, just drain
  auto give_up = [&]() {
    if (!dead && lane == 0) atomicExch(a.err, (int)a.launch_id);
    dead = true;
  };
  // Every wait for another workgroup is bounded by the same budget of real time (the constant
  // 100 MHz counter), measured from the first failed check of that wait.
  auto out_of_time = [&](unsigned long long& since) {
    const unsigned long long now = __builtin_amdgcn_s_memrealtime();
    if (since == ~0ull) since = now;
    return now - since >= a.wait_ticks;
  };
  if (blockIdx.x == 0 && tid == 0) st_result(a.err - 1, (int)a.launch_id, true);   // the launch the error word speaks of

  // The work of this wave as a list of segments (a sequence or a share of one); tile k of a segment is
  // row tile t0 + k * stride of sequence b.  Two partitions:
  //  * by context (default): the group's range of tiles [v0, v1) is cut at sequence boundaries and
  //    the waves take the tiles of a share round-robin; the waves' results are merged at the
  //    end of each share and the groups' partials by the projection.  Balanced for any lengths.
  //  * by sequence: every sequence is cut into a.by_sequence equal shares and wave slot g * NP + p
  //    takes shares round-robin; no merge inside the workgroup, one partial per share.  For batches
  //    whose shares fill the slots evenly (many short sequences).
  struct Seg { int b, t0, stride, ntl, len, pid; unsigned it0; const uint16_t* Kb; };   // it0: tiles of earlier segments
  constexpr bool by_seq = BYSEQ;
  int seg_b = by_seq ? g * NP + p : 0;
  unsigned seg_it = 0;                              // tiles this wave has been through so far
  if (has_work && !by_seq)
    while (prefix[seg_b + 1] <= v0) ++seg_b;
  auto next_segment = [&](Seg& sg) -> bool {
    if (by_seq) {
      const int shares = a.by_sequence;               // shares per sequence (equal runs of tiles)
      if (seg_b >= a.B * shares) return false;
      const int q = seg_b, b = q / shares, j = q - b * shares;
      seg_b += a.NG * NP;
      const int tiles_b = prefix[b + 1] - prefix[b], per = (tiles_b + shares - 1) / shares;
      sg.b = b; sg.t0 = j * per; sg.stride = 1; sg.pid = q;
      sg.len = lens_s[b];
      sg.Kb = a.K + (size_t)b * a.k_bstride;
      sg.ntl = max(0, min(per, tiles_b - j * per));
      sg.it0 = seg_it;
      seg_it += (unsigned)sg.ntl;
      return true;
    }
    for (; seg_b < a.B && prefix[seg_b] < v1; ++seg_b) {
      const int b = seg_b;
      const int s0 = max(v0, prefix[b]) - prefix[b];
      const int s1 = min(v1, prefix[b + 1]) - prefix[b];
      if (s0 >= s1) continue;
      sg.b = b; sg.pid = b + g;
      sg.t0 = s0 + p; sg.stride = NP;                 // this wave's tiles are s0+p, s0+p+NP, ...
      sg.len = lens_s[b];
      sg.Kb = a.K + (size_t)b * a.k_bstride;
      sg.ntl = max(0, (s1 - s0 - p + NP - 1) / NP);
      sg.it0 = seg_it;                                // tile k carries tag tag_base + it0 + k + 1
      seg_it += (unsigned)sg.ntl;
      ++seg_b;
      return true;
    }
    return false;
  };
  // End of a share in the by-context partition, all threads: sum the waves' accumulators
  // out of mbuf[wave][head][col] (one thread per four columns of a head) and write the group's
  // partial for this sequence.
  auto write_partial = [&](int pid) {
    const int oc4 = (tid & 31) * 4, oh0 = tid >> 5;  // four columns of heads oh0, oh0 + 16
    if (oc4 < uwc) {
#pragma unroll
      for (int jj = 0; jj < HP / 16; ++jj) {
        const int h = oh0 + 16 * jj;
        f32x4 osum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ww = 0; ww < NP; ++ww) osum += *reinterpret_cast<const f32x4*>(mbuf + ((size_t)ww * HP + h) * MERGE_PITCH + oc4);
        if (h < a.H) st_result4(a.Cpart + ((size_t)pid * a.H + h) * a.d + ucol0 + oc4, osum, fuse);
      }
    }
    if (u == 0 && tid < a.H) {
      const int t = tid >> 4, nn = tid & 15;
      float mall = NEG_INF, l = 0.f;
#pragma unroll
      for (int ww = 0; ww < NP; ++ww) {
        mall = fmaxf(mall, marr[ww][t][nn]);
        l += larr[ww][t][nn];
      }
      st_result(a.mpart + (size_t)pid * a.H + tid, mall, fuse);
      st_result(a.lpart + (size_t)pid * a.H + tid, l, fuse);
    }
  };

  if (has_work) {
    Seg sg;
    // rotary table: this lane's 4 column pairs start at pair li * 4 of the head
    const float* rope_lane = nullptr;
    const unsigned rope_pitch = (unsigned)(a.d_k / 2) * 8u;   // bytes per table row
    float w1c[4], w1s[4];                           // rotation by one position
    if constexpr (ROPE) {
      rope_lane = a.rope + (size_t)(col_active ? li : 0) * 8;
      const f32x4* r1 = reinterpret_cast<const f32x4*>(reinterpret_cast<const char*>(rope_lane) + (size_t)min(1, a.T - 1) * rope_pitch);
      const f32x4 v0 = r1[0], v1 = r1[1];
      w1c[0] = v0[0]; w1s[0] = v0[1]; w1c[1] = v0[2]; w1s[1] = v0[3];
      w1c[2] = v1[0]; w1s[2] = v1[1]; w1c[3] = v1[2]; w1s[3] = v1[3];
    }
    while (next_segment(sg)) {
      const int ntl = sg.ntl, len = sg.len;
      const uint16_t* Kb = sg.Kb;
      // query for this lane's 8 columns: requested here, used only after the first tiles have been
      // requested (the wait for it then overlaps theirs)
      const u32x4* qsrc = reinterpret_cast<const u32x4*>(a.q + (size_t)sg.b * a.d + (col_active ? mycol : 0));
      const u32x4 qraw0 = qsrc[0], qraw1 = qsrc[1];
      unsigned qh[4], ql[4];
      // (lanes without live columns re-read the unit's first columns: finite values that meet a zero
      //  query in the scores and accumulator rows nobody reads in the weighted sum)
      // Byte offset of element (row r, this lane's first column) from the sequence's start:
      //   (r / 32) * bandB + (r % 32) * rowB + lane_col_off
      // row-major cache: rowB = the row pitch; banded cache (32-row bands, head-major inside a band: a
      // head's 32 x d_k block is contiguous): rowB = d_k * 2 and the head's block offset joins the lane's.
      const unsigned bandB = TILE_ROWS * pitchB;
      const unsigned rowB = a.k_banded ? (unsigned)a.d_k * 2u : pitchB;
      const int lane_head = col_active ? myhead : u * a.hpu, lane_li = col_active ? li : 0;
      const unsigned lane_col_off = a.k_banded ? (unsigned)lane_head * TILE_ROWS * (unsigned)a.d_k * 2u + (unsigned)lane_li * 16u
                                               : (unsigned)(col_active ? mycol : ucol0) * 2u;
      const unsigned lane_off = (unsigned)(rg * RR) * rowB + lane_col_off;
      float mrun = NEG_INF;                           // running maximum of this lane's head (log2 domain)
      bf16x8 bq[4];                                   // B operands of the score MFMA (filled below, behind the first tile requests)
      // softmax state of the weighted sum and its accumulators; accl: sum of the weights (an all-ones A operand)
      float m[NT];
      f32x4 acc[8][NT], accl[NT];
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        m[t] = NEG_INF;
        accl[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i][t] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
      // Tiles travel HBM -> registers (PD register sets: one tile being scored, the other in flight)
      // -> LDS slot, where the same wave picks them up one step later.
      u32x4 ts[PD][8];
      f32x4 tr[PD][2];                                // ROPE: {cos, sin} x 4 pairs at the lane's first row of the tile
      // Every call issues the same number of loads on every path (also for k past the end of the segment,
      // where all rows collapse onto the last one and nobody uses the result): the compiler's s_waitcnt
      // for the next tile's registers is then exact.
      auto load_tile = [&](u32x4 (&t)[8], f32x4 (&r)[2], int k) {
        const int st = __builtin_amdgcn_readfirstlane(sg.t0 + k * sg.stride);
        if constexpr (ROPE) {
          const int row = min(st * TILE_ROWS + rg * 8, a.T - 1);
          const f32x4* rp = reinterpret_cast<const f32x4*>(reinterpret_cast<const char*>(rope_lane) + (size_t)row * rope_pitch);
          r[0] = rp[0];
          r[1] = rp[1];
        }
        if (k < ntl && (st + 1) * TILE_ROWS <= len) {
          // full tile: uniform row base + per-lane 32-bit offset
          const char* tb = reinterpret_cast<const char*>(Kb) + (size_t)st * bandB;
#pragma unroll
          for (int j = 0; j < 8; ++j)
            t[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(tb + (size_t)(j * RJ) * rowB + lane_off));
        } else {
          // last, partial tile (rows past the end re-read the last row; masked in the scores) or no tile
          const int r0 = st * TILE_ROWS + rg * RR;
          const char* cb = reinterpret_cast<const char*>(Kb) + lane_col_off;
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const int rr = max(min(r0 + j * RJ, len - 1), 0);
            t[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(cb + (size_t)(rr >> 5) * bandB + (size_t)(rr & 31) * rowB));
          }
        }
      };
      // ---- all heads' words of tile k: requested here, waited for in sum_step
      constexpr int GW = 2 * NT;                      // 16-byte words per lane and tile
      u32x4 gq[GW];
      auto gather = [&](int k) {
        const u32x4* base = team_ring + (size_t)((sg.it0 + (unsigned)k + 1u) & (EXCH_SLOTS - 1)) * (HP * 8) + (n * 4 + kg);
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
          for (int t = 0; t < NT; ++t) gq[c * NT + t] = ld_exch(base + (c * HP + t * 16) * 4);
      };
      auto pin_gq = [&]() {                           // (the asm loads' results, as far as the compiler is concerned)
        if constexpr (NT == 1) asm volatile("" : "+v"(gq[0]), "+v"(gq[1]) : : "memory");
        else asm volatile("" : "+v"(gq[0]), "+v"(gq[1]), "+v"(gq[2]), "+v"(gq[3]) : : "memory");
      };
      // ---- tile k out of its registers into its LDS slot (the tile that was there has been summed in the
      //      step before); tile k+2 requested into the registers
      auto park = [&](int k, auto SI) {
        u32x4 (&cur)[8] = ts[decltype(SI)::value];
        char* sl = myslots + (k & (NS - 1)) * SLOT_PITCH + wpos;
#pragma unroll
        for (int j = 0; j < 8; ++j) *reinterpret_cast<u32x4*>(sl + j * RJ * ROW_PITCH) = cur[j];
      };
      auto request = [&](int k, auto SI) { load_tile(ts[decltype(SI)::value], tr[decltype(SI)::value], k); };
      // ---- softmax numerators of the unit's heads from the 8 scores of a lane (row of score jj given by
      //      row_of), against the head's running maximum
      auto numerators = [&](int k, float (&sc)[8], unsigned (&pw)[4], auto&& row_of) {
        const int st = sg.t0 + k * sg.stride;
        if ((st + 1) * TILE_ROWS > len) {             // last, partial tile: rows past the end weigh nothing
#pragma unroll
          for (int j = 0; j < 8; ++j) sc[j] = (st * TILE_ROWS + row_of(j) < len) ? sc[j] : NEG_INF;
        }
        float tmax = fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])), fmaxf(fmaxf(sc[4], sc[5]), fmaxf(sc[6], sc[7])));
        tmax = max_over_row_groups(tmax);
        // The reference moves only when the maximum has grown by more than SOFTMAX_SLACK (log2 domain):
        // numerators stay below 2^SOFTMAX_SLACK, which costs bf16 and the fp32 sums nothing, and the
        // accumulators are rescaled rarely instead of at most early tiles.
        mrun = (tmax > mrun + SOFTMAX_SLACK) ? tmax : mrun;
        const float ref = (mrun == NEG_INF) ? 0.f : mrun;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const bf16x2 v = {(__bf16)__builtin_amdgcn_exp2f(sc[2 * i] - ref), (__bf16)__builtin_amdgcn_exp2f(sc[2 * i + 1] - ref)};
          pw[i] = __builtin_bit_cast(unsigned, v);
        }
      };
      // ---- scores of tile k on MFMA, from its LDS slot: S[row][n] = sum_c K[row][c] q_n[c], two M tiles of
      //      16 rows, four k-steps of 32 columns.  A lane ends up with rows mt*16 + rg*4 + r of column idx.
      auto score_mfma = [&](int k, unsigned (&pw)[4]) {
        const char* sl = myslots + (k & (NS - 1)) * SLOT_PITCH + spos;
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(sl + ks * 64);
          const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(sl + ks * 64 + 16 * ROW_PITCH);
          s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, bq[ks], s0, 0, 0, 0);
          s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, bq[ks], s1, 0, 0, 0);
        }
        float sc[8];
#pragma unroll
        for (int r = 0; r < 4; ++r) {                 // query hi + lo: neighbour columns
          sc[r] = dpp_add<0xB1>(s0[r]);
          sc[4 + r] = dpp_add<0xB1>(s1[r]);
        }
        numerators(k, sc, pw, [&](int jj) { return (jj >> 2) * 16 + rg * 4 + (jj & 3); });
      };
      // ---- scores of tile k with rotary keys, on the vector ALU from the tile's registers; a lane ends up
      //      with rows rg*8 + j of its head
      auto score_rotary = [&](int k, auto SI, unsigned (&pw)[4]) {
        u32x4 (&cur)[8] = ts[decltype(SI)::value];
        f32x4 (&rot)[2] = tr[decltype(SI)::value];
        float sc[8];
        float cc[4] = {rot[0][0], rot[0][2], rot[1][0], rot[1][2]};
        float ss[4] = {rot[0][1], rot[0][3], rot[1][1], rot[1][3]};
        // (-q2, q1) of every pair, same hi + lo split: rebuilt for every tile (three operations per word) so
        // that the eight registers are free during the rest of the step; the empty asm keeps the compiler
        // from hoisting them out of the loop again
        unsigned ph[4], pl[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          unsigned h = qh[c], l = ql[c];
          asm volatile("" : "+v"(h), "+v"(l));
          ph[c] = ((h >> 16) ^ 0x8000u) | (h << 16);
          pl[c] = ((l >> 16) ^ 0x8000u) | (l << 16);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          float sj = 0.f;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const unsigned kw = cur[j][c];             // (a scalar copy: bit_cast of a vector element picks lane 0)
            const bf16x2 kv = __builtin_bit_cast(bf16x2, kw);
            float da = __builtin_amdgcn_fdot2_f32_bf16(kv, __builtin_bit_cast(bf16x2, qh[c]), 0.f, false);
            da = __builtin_amdgcn_fdot2_f32_bf16(kv, __builtin_bit_cast(bf16x2, ql[c]), da, false);
            float db = __builtin_amdgcn_fdot2_f32_bf16(kv, __builtin_bit_cast(bf16x2, ph[c]), 0.f, false);
            db = __builtin_amdgcn_fdot2_f32_bf16(kv, __builtin_bit_cast(bf16x2, pl[c]), db, false);
            sj = fmaf(cc[c], da, sj);
            sj = fmaf(ss[c], db, sj);
            if (j < 7) {                              // on to the next row's position
              const float nc = fmaf(cc[c], w1c[c], -ss[c] * w1s[c]);
              ss[c] = fmaf(ss[c], w1c[c], cc[c] * w1s[c]);
              cc[c] = nc;
            }
          }
          sc[j] = sj;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {                 // sum over the head's lanes, all inside a 16-lane row
          if (lphp > 1) sc[j] = dpp_add<0xB1>(sc[j]);      // lane ^ 1   (a head spans lphp = 1, 2, 4, 8 or 16 lanes)
          if (lphp > 2) sc[j] = dpp_add<0x4E>(sc[j]);      // lane ^ 2
          if (lphp > 4) sc[j] = dpp_add<0x141>(sc[j]);     // other quad of the 8-lane half
          if (lphp > 8) sc[j] = dpp_add<0x140>(sc[j]);     // other half of the row
        }
        numerators(k, sc, pw, [&](int jj) { return rg * 8 + jj; });
      };
      // ---- publish tile k's words: {tag, running max, p0 p1, p2 p3} and {tag, 0, p4 p5, p6 p7} per row group
      auto publish = [&](int k, const unsigned (&pw)[4]) {
        const unsigned itk = sg.it0 + (unsigned)k + 1u;
        const unsigned tag = a.tag_base + itk;
        u32x4* ring = team_ring + (size_t)(itk & (EXCH_SLOTS - 1)) * (HP * 8);
        const int head = ROPE ? myhead : mhead;
        if (ROPE ? pub_lane : mpub_lane) {
          st_exch(ring + (head * 4 + rg), u32x4{tag, __float_as_uint(mrun), pw[0], pw[1]}, xl);
          st_exch(ring + ((HP + head) * 4 + rg), u32x4{tag, 0u, pw[2], pw[3]}, xl);
        }
      };
      // ---- the scoring half of a step: tile k parked, its numerators published
      auto score_tile = [&](int k, auto SI) {
        unsigned pw[4];
        if constexpr (ROPE) {
          score_rotary(k, SI, pw);
          park(k, SI);
        } else {
          park(k, SI);
          score_mfma(k, pw);
        }
        publish(k, pw);
      };
      // ---- weighted sum of tile k with the words gathered for it.  (k-slot jj of the operands is the row
      //      the numerators' jj stands for: rg*8 + jj with rotary keys, (jj / 4) * 16 + kg * 4 + jj % 4 otherwise.)
      //      HALF: the tile comes out of its slot in two halves of 64 columns (the first four and the last
      //      four columns of every lane), which keeps fewer registers live.
      auto tile_half = [&](int k, auto HALF, u32x4 (&am)[4]) {
        constexpr int hf = decltype(HALF)::value;
        const char* sl = myslots + (k & (NS - 1)) * SLOT_PITCH + (ROPE ? wpos : ppos) + hf * 8;
        unsigned lo[8], hi[8];                        // columns 4 hf + {0, 1} and 4 hf + {2, 3} of the lane's 8 rows
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
          const unsigned off = ROPE ? jj * ROW_PITCH : ((jj >> 2) * 16 + (jj & 3)) * ROW_PITCH;
          const auto v = *reinterpret_cast<const __attribute__((ext_vector_type(2))) unsigned*>(sl + off);
          lo[jj] = v[0];
          hi[jj] = v[1];
        }
#pragma unroll
        for (int jp = 0; jp < 4; ++jp) {                // (the 8 x 4 half of transpose8x8)
          am[0][jp] = __builtin_amdgcn_perm(lo[2 * jp + 1], lo[2 * jp], 0x05040100u);
          am[1][jp] = __builtin_amdgcn_perm(lo[2 * jp + 1], lo[2 * jp], 0x07060302u);
          am[2][jp] = __builtin_amdgcn_perm(hi[2 * jp + 1], hi[2 * jp], 0x05040100u);
          am[3][jp] = __builtin_amdgcn_perm(hi[2 * jp + 1], hi[2 * jp], 0x07060302u);
        }
      };
      // ---- every word of tile k must carry its tag; gather again while any is missing
      auto await_words = [&](int k) {
        const unsigned tag = a.tag_base + sg.it0 + (unsigned)k + 1u;
        pin_gq();
        unsigned long long since = ~0ull;
        for (;;) {
          unsigned bad = 0;
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            const unsigned bt = (gq[t][0] ^ tag) | (gq[NT + t][0] ^ tag);
            bad |= (heads_full || (t * 16 + n) < a.H) ? bt : 0u;
          }
          if (__all(bad == 0)) break;
          if (dead || out_of_time(since)) { give_up(); break; }
          __builtin_amdgcn_s_sleep(8);
          gather(k);
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          pin_gq();
        }
      };
      auto sum_finish = [&](int k, u32x4 (&am)[4]) {    // am: the first half, already out of the slot
        bf16x8 pb[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const bool live = heads_full || (t * 16 + n) < a.H;      // padded head: no weights at all
          const float mn = live ? __uint_as_float(gq[t][1]) : NEG_INF;
          const float ref = (mn == NEG_INF) ? 0.f : mn;            // all -inf so far: exp2(-inf - 0) = 0
          const float alpha = __builtin_amdgcn_exp2f(m[t] - ref);
          m[t] = mn;
          const u32x4 pw = live ? u32x4{gq[t][2], gq[t][3], gq[NT + t][2], gq[NT + t][3]} : u32x4{0u, 0u, 0u, 0u};
          pb[t] = __builtin_bit_cast(bf16x8, pw);
          if (__any(alpha != 1.f)) {
            accl[t] *= alpha;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i][t] *= alpha;
          }
        }
        const u32x4 ones_bits = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
        const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_bits);
#pragma unroll
        for (int t = 0; t < NT; ++t) accl[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[t], accl[t], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const bf16x8 av = __builtin_bit_cast(bf16x8, am[i]);
#pragma unroll
          for (int t = 0; t < NT; ++t)
            acc[i][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, pb[t], acc[i][t], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);            // (the second half's registers only after the first half's are dead)
        tile_half(k, std::integral_constant<int, 1>{}, am);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const bf16x8 av = __builtin_bit_cast(bf16x8, am[i]);
#pragma unroll
          for (int t = 0; t < NT; ++t)
            acc[4 + i][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, pb[t], acc[4 + i][t], 0, 0, 0);
        }
      };
      // One step (k >= 1).  Tile k is scored and published first; only then are the words of tile k-1
      // requested (every workgroup of the group published them a scoring time ago), and behind them
      // tile k+2 (LOADS_PER_TILE loads, the only vector-memory operations younger than the gather when it
      // is waited for).  The tile comes out of its slot while the words travel.  (Requesting the words
      // before the scoring instead, and tile k+2 only after they have been checked, was measured: no
      // faster at 8 tiles per wave, 4 % slower on long sequences.)
      constexpr int LOADS_PER_TILE = ROPE ? 10 : 8;
      auto step = [&](int k, auto SI) {
        u32x4 am[4];
        score_tile(k, SI);
        gather(k - 1);
        request(k + PD, SI);
        tile_half(k - 1, std::integral_constant<int, 0>{}, am);
        if constexpr (ROPE) asm volatile("s_waitcnt vmcnt(10)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        static_assert(LOADS_PER_TILE == (ROPE ? 10 : 8), "the wait above counts the loads of one tile");
        await_words(k - 1);
        sum_finish(k - 1, am);
      };

      f32x4 qx[4][2];                                 // the query columns behind bq, as loaded
      bool qlive[4];
      if constexpr (!ROPE) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const int C = ks * 4 + rg, hq = C / lphp, lq = C % lphp;
          qlive[ks] = lq < a.lph && hq < a.hpu && u * a.hpu + hq < a.H && (idx >> 1) == hq;
          const f32x4* src = reinterpret_cast<const f32x4*>(a.q + (size_t)sg.b * a.d + (qlive[ks] ? (u * a.hpu + hq) * a.d_k + lq * 8 : 0));
          qx[ks][0] = src[0];
          qx[ks][1] = src[1];
        }
      }
#pragma unroll
      for (int k = 0; k < PD; ++k) load_tile(ts[k], tr[k], k);
      // B operands of the score MFMA: k-step ks covers chunks ks*4 .. ks*4+3 of the unit; this lane holds
      // chunk ks*4 + rg of column n = idx: the head's query (pre-scaled, bf16 hi or lo) where the chunk
      // belongs to that head, zero elsewhere.  (Requested ahead of the first tiles, converted behind
      // their requests: the wait for it then overlaps theirs.)
      if constexpr (!ROPE) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
          const f32x4 x0 = qx[ks][0], x1 = qx[ks][1];
          const bool live = qlive[ks];
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const float f = live ? (i < 4 ? x0[i] : x1[i - 4]) * a.qscale : 0.f;
            const __bf16 h = (__bf16)f;
            bq[ks][i] = (idx & 1) ? (__bf16)(f - (float)h) : h;
          }
        }
      }
      // the query, pre-scaled (log2 domain), split into bf16 hi + lo pairs so that the dot products run
      // on v_dot2c_f32_bf16 without losing the fp32 query
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const unsigned r0 = c < 2 ? qraw0[2 * c] : qraw1[2 * c - 4], r1 = c < 2 ? qraw0[2 * c + 1] : qraw1[2 * c - 3];
        const float f0 = col_active ? __uint_as_float(r0) * a.qscale : 0.f;
        const float f1 = col_active ? __uint_as_float(r1) * a.qscale : 0.f;
        const __bf16 h0 = (__bf16)f0, h1 = (__bf16)f1;
        const bf16x2 hi = {h0, h1};
        const bf16x2 lo = {(__bf16)(f0 - (float)h0), (__bf16)(f1 - (float)h1)};
        qh[c] = __builtin_bit_cast(unsigned, hi);
        ql[c] = __builtin_bit_cast(unsigned, lo);
      }
      {
        using S0 = std::integral_constant<int, 0>;
        using S1 = std::integral_constant<int, 1>;
        // (the request is unconditional: a path into the loop without it would make the compiler wait for
        //  every outstanding load at the top of each step)
        if (ntl > 0) score_tile(0, S0{});
        request(PD, S0{});
        // Whole rounds of PD steps without a condition between them (a step that may be skipped
        // inside the loop would make the compiler's waits for the tile registers conservative).
        int k = 1;
        for (; k + PD <= ntl; k += PD) {
          step(k, S1{});
          step(k + 1, S0{});
        }
        if (k < ntl) step(k, S1{});
        // the last tile: nothing left to score while its words travel
        if (ntl > 0) {
          u32x4 am[4];
          gather(ntl - 1);
          tile_half(ntl - 1, std::integral_constant<int, 0>{}, am);
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          await_words(ntl - 1);
          sum_finish(ntl - 1, am);
        }
      }

      // ---- end of this sequence's share ---------------------------------------------------------------
      if (by_seq) {
        // the whole share was this wave's: its partial needs no merge.  A lane holds 8 consecutive columns
        // of a head per accumulator row; stored from there, an instruction writes 64 16-byte pieces into 64
        // different cache lines (7 of 71 us at 64 sequences of 1500 rows).  So head tile t goes through the
        // wave's (idle) slot t and leaves with a head's columns on consecutive lanes.
        constexpr int OP = 128 + 4;                     // floats per head row in the slot (padding: no bank conflicts)
        static_assert(16 * OP * 4 <= SLOT_PITCH && NT <= NS, "a head tile's block must fit one slot");
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          float* const ob = reinterpret_cast<float*>(myslots + t * SLOT_PITCH) + n * OP;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            if (ocol[r] < 0) continue;
            *reinterpret_cast<f32x4*>(ob + ocol[r]) = f32x4{acc[0][t][r], acc[1][t][r], acc[2][t][r], acc[3][t][r]};
            *reinterpret_cast<f32x4*>(ob + ocol[r] + 4) = f32x4{acc[4][t][r], acc[5][t][r], acc[6][t][r], acc[7][t][r]};
          }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // (LDS operations of one wave complete in order)
        {
          // head hl of the block on lanes 32 (hl % 2) .. +31, four columns per lane; two heads per instruction
          const int c4 = (lane & 31) * 4;
          const float* src = reinterpret_cast<const float*>(myslots) + (lane >> 5) * OP + c4;
          float* dst = a.Cpart + ((size_t)sg.pid * a.H + (lane >> 5)) * a.d + ucol0 + c4;
          const int nh = min(a.H, HP);
#pragma unroll 1
          for (int hl = lane >> 5; hl < nh; hl += 2) {
            const int t = hl >> 4;
            const f32x4 v = *reinterpret_cast<const f32x4*>(src + (t * (SLOT_PITCH / 4 - 16 * OP)));
            if (c4 < uwc) st_result4(dst, v, fuse);
            src += 2 * OP;
            dst += 2 * (size_t)a.d;
          }
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // (the next share parks its tiles in these slots)
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const int h = t * 16 + n;
          if (u == 0 && kg == 0 && h < a.H) {
            st_result(a.mpart + (size_t)sg.pid * a.H + h, m[t], fuse);
            st_result(a.lpart + (size_t)sg.pid * a.H + h, accl[t][0], fuse);
          }
        }
        continue;
      }
      // ---- by context: merge the waves and write one partial (every wave of the workgroup walks the
      //      same shares, so all of them meet at these barriers) -------------------------------------
      __syncthreads();                                // every slot is idle from here on
      if (kg == 0) {
#pragma unroll
        for (int t = 0; t < NT; ++t) marr[p][t][n] = m[t];
      }
      __syncthreads();
      {
        // accumulators -> mbuf[wave][head][col], in MFMA layout, scaled to the maximum over the waves
        float wsc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          float mall = NEG_INF;
#pragma unroll
          for (int ww = 0; ww < NP; ++ww) mall = fmaxf(mall, marr[ww][t][n]);
          wsc[t] = (m[t] == NEG_INF) ? 0.f : exp2f(m[t] - mall);
          if (kg == 0) larr[p][t][n] = accl[t][0] * wsc[t];   // every accumulator row holds the same sum
        }
        float* mine = mbuf + (size_t)p * HP * MERGE_PITCH + n * MERGE_PITCH;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (ocol[r] < 0) continue;
#pragma unroll
          for (int t = 0; t < NT; ++t) {
            f32x4* dst = reinterpret_cast<f32x4*>(mine + t * 16 * MERGE_PITCH + ocol[r]);
            dst[0] = f32x4{acc[0][t][r], acc[1][t][r], acc[2][t][r], acc[3][t][r]} * wsc[t];
            dst[1] = f32x4{acc[4][t][r], acc[5][t][r], acc[6][t][r], acc[7][t][r]} * wsc[t];
          }
        }
      }
      __syncthreads();
      write_partial(sg.pid);
      __syncthreads();                                // the slots are reused by the next share
    }
  }
  if (!fuse) return;

  // ========================= single-launch mode: merge + projection ===============================
  // This workgroup's partials are out (write-through stores, waited for) before its arrival flag.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (tid == 0) st_result(reinterpret_cast<int*>(a.flags) + blockIdx.x, (int)a.launch_id, true);
  const int wg = blockIdx.x;
  if (wg >= a.proj.H * a.proj.csw) return;
  // (everything of the stream phase is over in this workgroup: its LDS is reused)
  ProjShared<1>& psm = *reinterpret_cast<ProjShared<1>*>(sbuf);
  project_work<1, true, false>(a.proj, wg / a.proj.csw, wg % a.proj.csw, 0, prefix, psm, red, [&]() {
    // every workgroup's partials must be out: all arrival flags carry this launch's id
    if (wu == 0) {
      unsigned long long since = ~0ull;
      for (;;) {
        // all flags of a poll in one round trip (a chain of "ok && load" would take one trip per 64 flags)
        unsigned seen[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
          seen[j] = __hip_atomic_load(a.flags + min(lane + 64 * j, (int)gridDim.x - 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const bool ok = seen[0] == a.launch_id && seen[1] == a.launch_id && seen[2] == a.launch_id && seen[3] == a.launch_id;
        static_assert(FUSED_MAX_GRID <= 256, "four flags per lane cover the grid");
        if (__all(ok)) break;
        if (dead || out_of_time(since)) { give_up(); break; }
        __builtin_amdgcn_s_sleep(4);
      }
    }
    __syncthreads();
  });
}

// Records which XCD each workgroup of a 256-workgroup launch runs on.
__global__ __launch_bounds__(512) void xcc_probe_kernel(unsigned* out) {
  const unsigned xcc = __builtin_amdgcn_s_getreg((31 << 11) | 20);   // HW_REG_XCC_ID
  if (threadIdx.x == 0) out[blockIdx.x] = xcc & 0xf;
  for (int i = 0; i < 200; ++i) __builtin_amdgcn_s_sleep(10);        // stay resident while the rest start
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
bool fused_geometry(int B, int H, int T, int d, FusedGeom* g) {
  if (H < 1 || d % H != 0) return false;
  const int d_k = d / H;
  if (d_k % 8 != 0 || d_k < 16 || d_k > 128 || H > 32 || B > FUSED_MAX_B) return false;   // (16 score columns hold 8 heads of a unit, hi + lo)
  g->lph = d_k / 8;
  int lphp = 1;
  while (lphp < g->lph) lphp <<= 1;
  g->lphp = lphp;
  g->hpu = 16 / lphp;
  g->G = (H + g->hpu - 1) / g->hpu;
  g->NT = H <= 16 ? 1 : 2;
  g->NP = FUSED_WAVES;
  const int cus = FUSED_MAX_GRID;
  if (g->G > cus) return false;
  if (g->G <= 32) {
    g->gpx = 32 / g->G;
    if (g->gpx > 8) g->gpx = 8;                     // at most PROJ_MAX_PARTS groups
    g->NG = 8 * g->gpx;
    g->grid = cus;
  } else {
    g->gpx = 0;
    g->NG = cus / g->G;
    g->grid = g->NG * g->G;
  }
  g->nparts = B + g->NG - 1;
  return true;
}

// True when workgroups i and j of a 256-workgroup launch share an XCD whenever i % 8 == j % 8: a probe
// launch on `st` that records each workgroup's XCD into `dev_buf` (device memory, 256 unsigned), read
// back with a blocking copy.  The caller caches the answer per device.
bool probe_xcd_round_robin(unsigned* dev_buf, hipStream_t st) {
  unsigned h[256];
  hipLaunchKernelGGL(xcc_probe_kernel, dim3(256), dim3(512), 0, st, dev_buf);
  bool ok = hipMemcpyAsync(h, dev_buf, sizeof(h), hipMemcpyDeviceToHost, st) == hipSuccess &&
            hipStreamSynchronize(st) == hipSuccess;
  if (ok)
    for (int i = 8; i < 256 && ok; ++i) ok = h[i] == h[i & 7];
  if (ok)
    for (int i = 1; i < 8 && ok; ++i)
      for (int j = 0; j < i; ++j) ok = ok && h[i] != h[j];
  (void)hipGetLastError();
  return ok;
}

// Workgroups of the stream kernel one compute unit can hold at once (0 on error): the launch is only
// safe when all of its workgroups are resident together.
int fused_blocks_per_cu(const FusedGeom& g, bool rope) {
  int n = 0;
  auto ask = [&](auto nt, auto rp, auto lp) {                 // (the smaller figure of the two partitions' instantiations)
    int n0 = 0, n1 = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n0, fused_stream_kernel<decltype(nt)::value, decltype(rp)::value, decltype(lp)::value, false>,
                                                     g.NP * 64, 0) != hipSuccess) { n0 = 0; (void)hipGetLastError(); }
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n1, fused_stream_kernel<decltype(nt)::value, decltype(rp)::value, decltype(lp)::value, true>,
                                                     g.NP * 64, 0) != hipSuccess) { n1 = 0; (void)hipGetLastError(); }
    n = n0 < n1 ? n0 : n1;
  };
  auto with_lphp = [&](auto nt, auto rp) {
    if (g.lphp == 16) ask(nt, rp, std::integral_constant<int, 16>{});
    else if (g.lphp == 8) ask(nt, rp, std::integral_constant<int, 8>{});
    else ask(nt, rp, std::integral_constant<int, 0>{});
  };
  auto with_rope = [&](auto nt) {
    if (rope) with_lphp(nt, std::true_type{});
    else with_lphp(nt, std::false_type{});
  };
  if (g.NT == 1) with_rope(std::integral_constant<int, 1>{});
  else with_rope(std::integral_constant<int, 2>{});
  return n;
}

// By-sequence partition: how many equal shares to cut every sequence into so that the shares fill
// the wave slots (groups x waves) evenly (1..4), or 0 to keep the balanced by-context partition.  Ragged
// batches qualify only with many shares per slot.
int fused_by_sequence(const FusedGeom& g, int B, bool ragged) {
  const long slots = (long)g.NG * FUSED_WAVES;
  int best = 0;
  double best_waste = 1.13;                           // at most 13 % idle slot-time
  for (int s = 1; s <= 4; ++s) {
    const long shares = (long)B * s, rounds = (shares + slots - 1) / slots;
    const double waste = (double)(rounds * slots) / (double)shares;
    if (ragged && shares < 4 * slots) continue;
    if (waste < best_waste - 0.04) { best = s; best_waste = waste; }
  }
  return best;
}

size_t fused_exch_bytes(const FusedGeom& g) {
  // per team and ring slot: two 16-byte words for each (padded head, row group of 8)
  return (size_t)g.NG * g.NP * EXCH_SLOTS * (g.NT * 16) * 8 * 16;
}

void launch_fused_stream(const FusedGeom& g, const FusedArgs& a, hipStream_t st) {
  dim3 grid(g.grid), block(g.NP * 64);
  auto go = [&](auto nt, auto rope, auto lphp) {
    if (a.by_sequence)
      hipLaunchKernelGGL((fused_stream_kernel<decltype(nt)::value, decltype(rope)::value, decltype(lphp)::value, true>), grid, block, 0, st, a);
    else
      hipLaunchKernelGGL((fused_stream_kernel<decltype(nt)::value, decltype(rope)::value, decltype(lphp)::value, false>), grid, block, 0, st, a);
  };
  auto with_lphp = [&](auto nt, auto rope) {
    if (g.lphp == 16) go(nt, rope, std::integral_constant<int, 16>{});
    else if (g.lphp == 8) go(nt, rope, std::integral_constant<int, 8>{});
    else go(nt, rope, std::integral_constant<int, 0>{});
  };
  auto with_rope = [&](auto nt) {
    if (a.rope) with_lphp(nt, std::true_type{});
    else with_lphp(nt, std::false_type{});
  };
  if (g.NT == 1) with_rope(std::integral_constant<int, 1>{});
  else with_rope(std::integral_constant<int, 2>{});
}

// Sequences per workgroup of the projection, in MFMA N tiles of 16 (1, 2 or 4).  One tile keeps the
// kernel out of register spills and gives more workgroups; it costs one more pass over W_KV per 16
// sequences, which is only worth it while those passes stay small.
int proj_batch_tiles(int B, int rows, int e, int H) {
  if (B <= 16) return 1;
  const long w_bytes = (long)rows * e * 2;
  // One tile of 16 sequences per workgroup (no register spills, most workgroups) as long as one round of
  // workgroups, one per CU, covers every (head, batch chunk); W is read once per batch chunk (mostly from
  // L2), which bounds the number of chunks.  Measured at B = 64, H = 20: 14.8 us against 19.1 us with two tiles.
  for (int nbt = 1; nbt <= 2; nbt *= 2) {            // (four batch tiles per workgroup measured slower than two rounds)
    const long chunks = (B + 16 * nbt - 1) / (16 * nbt);
    if ((long)H * chunks <= 256 && w_bytes * chunks <= (64L << 20)) return nbt;
  }
  if (w_bytes * ((B + 15) / 16) <= (64L << 20)) return 1;
  return B <= 32 ? 2 : 4;
}

int proj_row_splits(int H, int rows, int e, int B) {
  // one 32-row tile of W per wave (8 waves = 256 rows per workgroup) unless that makes more
  // workgroups than CUs
  const int per = 16 * proj_batch_tiles(B, rows, e, H);
  const int zb = (B + per - 1) / per;
  int csw = (rows + 8 * TILE_ROWS - 1) / (8 * TILE_ROWS);
  const int cap = 256 / (H * zb);                     // one workgroup per CU: a single round
  if (csw > cap) csw = cap;
  if (csw < 1) csw = 1;
  return csw;
}

int proj_rows_per_split(int rows, int csw) {
  return ((rows + csw - 1) / csw + TILE_ROWS - 1) / TILE_ROWS * TILE_ROWS;
}

void launch_project_mfma(ProjArgs a, hipStream_t st) {
  const int nbt = proj_batch_tiles(a.B, a.rows, a.e, a.H);
  a.crows = proj_rows_per_split(a.rows, a.csw);
  dim3 grid(a.H, a.csw, (a.B + 16 * nbt - 1) / (16 * nbt)), block(512);
  if (nbt == 1) hipLaunchKernelGGL((project_mfma_kernel<1, false>), grid, block, 0, st, a);
  else if (nbt == 2) hipLaunchKernelGGL((project_mfma_kernel<2, false>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((project_mfma_kernel<4, false>), grid, block, 0, st, a);
}

// out_m = x W_m for a.nmat matrices in one launch (a.Cpart = x, a.csw from dense_row_splits).
void launch_dense_mfma(ProjArgs a, hipStream_t st) {
  const int nbt = proj_batch_tiles(a.B, a.rows, a.e, a.H * a.nmat);
  a.crows = proj_rows_per_split(a.rows, a.csw);
  a.mode = 2;
  dim3 grid(a.H * a.nmat, a.csw, (a.B + 16 * nbt - 1) / (16 * nbt)), block(512);
  if (nbt == 1) hipLaunchKernelGGL((project_mfma_kernel<1, true>), grid, block, 0, st, a);
  else if (nbt == 2) hipLaunchKernelGGL((project_mfma_kernel<2, true>), grid, block, 0, st, a);
  else hipLaunchKernelGGL((project_mfma_kernel<4, true>), grid, block, 0, st, a);
}

int dense_row_splits(int H, int nmat, int rows, int e, int B) {
  return proj_row_splits(H * nmat, rows, e, B);
}

}  // namespace slim
