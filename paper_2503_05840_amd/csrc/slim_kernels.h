// Internal launch interface between the C-ABI layer (slim_api.hip) and the kernel files.
// Everything here is device-pointer based; shapes have been validated by the caller.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace slim {

constexpr int DT_F32 = 0;
constexpr int DT_BF16 = 1;

inline int vec_elems(int dtype) { return dtype == DT_BF16 ? 8 : 4; }   // elements per 16-byte vector
inline int elem_bytes(int dtype) { return dtype == DT_BF16 ? 2 : 4; }

// ---- generic vector-ALU kernels (kernels_generic.hip) ------------------------------------------

// S[b][h][r] = scale * sum_j q[b][h*d_k + j] * M[b][r][h*d_k + j]   for r < rows_b
// (attention scores against a K-cache, eq. 2; also q_h W_K,h^T for the X-cache scheme with
//  M := W_K, rows := d_model, m_bstride := 0).  rope: nullable [rows][d_k/2] {cos, sin}; when set,
// row r is rotated by position r before the dot product (RoPE appendix, option 1).
void launch_head_scores(int dtype, const float* q, long q_bstride, const void* M, long m_bstride,
                        long row_pitch, const int32_t* rows_per_b, int rows, int e, int H, int d_k,
                        float scale, float* S, long s_bstride, const float* rope, int B, hipStream_t st);

// S[b][h][t] = scale * sum_c qt[b][h][c] * X[b][t][c]   (X-cache scores, Fig. 4)
void launch_dense_scores(int dtype, const float* qt, const void* X, long x_bstride, int d_model,
                         const int32_t* seq_lens, int T, int H, float scale, float* S, int B,
                         hipStream_t st);

// Per (b, split): m = max_t S, l = sum_t exp(S - m), Cpart[h][c] = sum_t exp(S - m) M[t][c]
void launch_weighted_sum(int dtype, const float* S, const void* M, long m_bstride, int width,
                         const int32_t* seq_lens, int T, int H, int nsplit, float* Cpart,
                         float* mpart, float* lpart, int B, hipStream_t st);

// Cn[b][h][c] = sum_s e^{m_s - m} Cpart_s[h][c] / sum_s e^{m_s - m} l_s
void launch_combine(const float* Cpart, const float* mpart, const float* lpart, int nsplit,
                    int H, int width, float* Cn, int B, hipStream_t st);

// out[b][n] = sum_c Cn[b][n / d_k][c] * W[c][n],  W row-major [rows][e]
void launch_project(int dtype, const float* Cn, const void* W, int rows, int e, int H, int d_k,
                    float* out, int B, hipStream_t st);

// New token rows into the caches at row len_b - 1: K <- knew (rotated to that position when rope and
// rotate_k), V <- vnew (nullable: no V-cache); with rope, q [B][d] is rotated in place as well.
void launch_append(int dtype, const float* knew, const float* vnew, void* K, void* V, long bstride,
                   const int32_t* seq_lens, int T, int d, int d_k, const float* rope, float* q, int rotate_k,
                   int B, hipStream_t st);
void launch_zero_ints(int* p, int n, hipStream_t st);
// Plain streaming read of `bytes` (measurement only).
void launch_read_probe(const void* buf, size_t bytes, hipStream_t st);

// Vanilla K+V decode: partial (m, l, acc) per (b, split, head) then a merge.
int vanilla_heads_per_wave(int dtype, int d_k);   // heads a wave of the packed bf16 kernel covers (0: plain kernel)
void launch_vanilla(int dtype, const float* q, const void* K, const void* V, long bstride,
                    const int32_t* seq_lens, int T, int H, int d_k, int nsplit, float* acc,
                    float* mpart, float* lpart, float* out, int B, hipStream_t st);

// ---- bf16 fast path (kernels_bf16.hip) -----------------------------------------------------------
constexpr int TILE_ROWS = 32;        // cache rows per wave tile
constexpr int EXCH_SLOTS = 16;       // ring depth of the score exchange (a power of two >= 2 * FUSED_SLOTS)
constexpr int FUSED_MAX_B = 1024;    // sequences per call the fast path handles
constexpr int FUSED_MAX_GRID = 256;  // workgroups of a stream-kernel launch at most (one per compute unit)
constexpr int FUSED_WAVES = 8;       // waves per workgroup of the stream kernel, each with tiles of its own
constexpr int FUSED_SLOTS = 2;       // LDS landing slots (8 KB tiles) per wave
constexpr int FUSED_AHEAD = 2;       // register sets of a wave: one tile being scored, the other in flight
constexpr int PROJ_MAX_PARTS = 64;   // partials per sequence the projection merges

struct FusedGeom {
  int lph, lphp, hpu;   // active lanes per head (d_k/8), lanes reserved per head, heads per unit
  int G, NG, gpx;       // column units per group, groups, groups per XCD (0 = not packed)
  int NT, NP, grid, nparts;   // MFMA head tiles, waves per workgroup
};

struct ProjArgs {
  const float* Cpart; const float* mpart; const float* lpart;
  const uint16_t* W;                  // [rows][e] bf16
  float* out; float* outpart;         // [B][e], [csw][B][e]
  int* counters; const int* err; unsigned launch_id;
  const int32_t* seq_lens;
  int B, T, H, d_k, rows, e;
  int NG, nsplit, mode;               // mode 0: partials laid out by the stream kernel; 1: [b][nsplit]
  float mscale;                       // 1 for log2-domain maxima, log2(e) for natural-log ones
  int csw, crows;                     // row splits of W across workgroups, rows per split
  // Dense products (launch_dense_mfma): Cpart = x [B][rows], out_m = x W_m for nmat matrices.
  // role 0: fp32 result.  The new token's rows (it sits at row / position seq_lens[b] - 1):
  // role 1: query, fp32, rotated to that position when rope is set; role 2: key row into Kc (rotated
  // when rope and rotate_k); role 3: value row into Vc.
  int nmat;
  const uint16_t* Wm[3]; float* outm[3]; int role[3];
  uint16_t* Kc; uint16_t* Vc; long c_bstride;
  int k_banded;                       // Kc is a banded cache (see FusedArgs::k_banded)
  const float* rope; int rotate_k;
};

struct FusedArgs {
  const float* q;
  const uint16_t* K;
  long k_bstride;
  int k_banded;                       // 0: [t][d] row-major per sequence; 1: [t / 32][H][32][d_k] (32-row bands, head-major)
  const int32_t* seq_lens;
  int T, B, H, d, d_k;
  int G, NG, gpx, lph, lphp, hpu;
  float qscale;                       // log2(e) / sqrt(d_k): scores live in the log2 domain
  unsigned long long* exch;           // [NG][NP][EXCH_SLOTS][2][16*NT][4] 16-byte words {tag, max, 4 bf16 weights}
  unsigned tag_base, launch_id;
  unsigned long long wait_ticks;      // budget of every wait for another workgroup, in ticks of the 100 MHz real-time counter
  float* Cpart;                       // [nparts][H][d]
  float* mpart;                       // [nparts][H]  running max, log2 domain
  float* lpart;                       // [nparts][H]
  int* err;                           // set to launch_id when a wait timed out; err[-1] receives launch_id at the start
  int* counters;                      // arrival counters of the projection, zeroed here
  int ncounters;
  int xcd_local;                      // 1: a group's workgroups share an XCD, the exchange stays in its L2
  // Single-launch mode: once all workgroups have written their partials (arrival flags, tagged
  // with launch_id), each takes a (head, row split) share of the merge + projection.
  const float* rope;                  // nullable [T][d_k/2] {cos, sin}: rotate key rows by position for the scores
  int by_sequence;                    // > 0: by-sequence partition with this many shares per sequence
  int fuse;
  unsigned* flags;                    // [grid]
  ProjArgs proj;                      // csw * H <= grid, B <= 16
};


bool fused_geometry(int B, int H, int T, int d, FusedGeom* g);
int fused_by_sequence(const FusedGeom& g, int B, bool ragged);
size_t fused_exch_bytes(const FusedGeom& g);
bool probe_xcd_round_robin(unsigned* dev_buf, hipStream_t st);
int fused_blocks_per_cu(const FusedGeom& g, bool rope);
void launch_fused_stream(const FusedGeom& g, const FusedArgs& a, hipStream_t st);
int proj_batch_tiles(int B, int rows, int e, int H);
int proj_row_splits(int H, int rows, int e, int B);
int proj_rows_per_split(int rows, int csw);
void launch_project_mfma(ProjArgs a, hipStream_t st);
int dense_row_splits(int H, int nmat, int rows, int e, int B);
void launch_dense_mfma(ProjArgs a, hipStream_t st);

// ---- bf16 fast path of the X-cache scheme (kernels_xcache.hip) -------------------------------------
bool xcache_fast_ok(int dtype, int H, int d_model, int d_k);
int xcache_splits(int B, int H, int T, int d_model);
void launch_xq_tilde(const float* q, const void* Wk, float* qt, int B, int H, int d_k, int d_model, int e,
                     float scale, int* counters, int ncounters, hipStream_t st);
void launch_xscores(const float* qt, const void* X, long x_bstride, const int32_t* seq_lens, int T, int H,
                    int d_model, float* S, int B, hipStream_t st);
bool xfused_ok(int d_model);                 // one pass over X instead of xscores + xweighted
int xfused_splits(int B, int H, int T, int d_model);
void launch_xfused(const float* qt, const void* X, long x_bstride, const int32_t* seq_lens, int T, int H, int d_model,
                   int nsplit, float* Cpart, float* mpart, float* lpart, int B, hipStream_t st);
void launch_xweighted(const float* S, const void* X, long x_bstride, const int32_t* seq_lens, int T, int H,
                      int d_model, int nsplit, float* Cpart, float* mpart, float* lpart, int B, hipStream_t st);

}  // namespace slim
