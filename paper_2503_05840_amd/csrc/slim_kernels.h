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
//  M := W_K, rows := d_model, m_bstride := 0).
void launch_head_scores(int dtype, const float* q, long q_bstride, const void* M, long m_bstride,
                        long row_pitch, const int32_t* rows_per_b, int rows, int e, int H, int d_k,
                        float scale, float* S, long s_bstride, int B, hipStream_t st);

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

// Vanilla K+V decode: partial (m, l, acc) per (b, split, head) then a merge.
void launch_vanilla(int dtype, const float* q, const void* K, const void* V, long bstride,
                    const int32_t* seq_lens, int T, int H, int d_k, int nsplit, float* acc,
                    float* mpart, float* lpart, float* out, int B, hipStream_t st);

}  // namespace slim
