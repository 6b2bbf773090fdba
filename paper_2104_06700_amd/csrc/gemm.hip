// Dense update of a GNN layer (the MLP step that follows the aggregation, Section 6.3 "Memory"):
//
//   C[m, n] = act( sum_k opA(A)[m, k] * opB(B)[k, n] + bias[n] )
//
// fp32 in, fp32 out, on the matrix cores: v_mfma_f32_32x32x2_f32 multiplies exact fp32 products and
// accumulates in fp32, so the result meets the same tolerance as the aggregation.  A workgroup of
// four wavefronts owns a 128 x 128 tile of C; each wavefront a 64 x 64 quarter as 2 x 2 MFMA
// tiles.  A and B tiles of 16 k-steps are staged through LDS k-major ([k][m] and [k][n]), so that
// the 32 lanes of an MFMA operand read consecutive words; the global loads follow whichever
// direction of the operand is contiguous.  The reduction over a very long k (the weight gradient:
// k = number of vertices) is split over blockIdx.z into partial tiles that a second kernel adds in
// order (deterministic, no atomics).
#include "common.h"

namespace {

constexpr int BM = 128, BN = 128, BK = 16;
constexpr int PAD = 4;  // row stride BM + PAD: k-rows start 4 banks apart
constexpr int kThreads = 256;

typedef float float16v __attribute__((ext_vector_type(16)));

struct GemmArgs {
    const float *A;
    const float *B;
    float *C;           // or the partial buffer when n_split > 1
    const float *bias;  // [N] or nullptr
    int64_t sam, sak;   // element strides of opA(A)[m, k]
    int64_t sbk, sbn;   // element strides of opB(B)[k, n]
    int64_t ldc;
    int64_t M, N, K;
    int64_t k_per_split;
    int32_t relu;
    int32_t n_split;
};

// Stages a [rows x BK] tile of an operand into LDS as tile[k][r].  X(r, k) = base[r * sr + k * sk].
// K_CONTIG: sk == 1 (threads run along k with 16-byte loads when aligned), else sr == 1.
template <bool K_CONTIG>
__device__ __forceinline__ void stage_tile(float (*tile)[BM + PAD], const float *__restrict__ base, int64_t sr, int64_t sk,
                                           int64_t r0, int64_t r_end, int64_t k0, int64_t k_end, bool vec_ok) {
    const int t = threadIdx.x;
    if (K_CONTIG) {
        // 128 rows x 16 k = 512 quads of 4 k; thread t takes quads t and t + 256
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int q = t + h * kThreads;
            const int r = q >> 2, kq = (q & 3) * 4;
            const int64_t gr = r0 + r, gk = k0 + kq;
            float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (gr < r_end) {
                const float *p = base + gr * sr + gk;
                if (vec_ok && gk + 3 < k_end) {
                    const float4 x = *reinterpret_cast<const float4 *>(p);
                    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (gk + i < k_end) v[i] = p[i];
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) tile[kq + i][r] = v[i];
        }
    } else {
        // rows contiguous: 16 k x 32 quads of 4 rows; thread t takes quads t and t + 256
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int q = t + h * kThreads;
            const int k = q >> 5, rq = (q & 31) * 4;
            const int64_t gk = k0 + k, gr = r0 + rq;
            float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (gk < k_end) {
                const float *p = base + gk * sk + gr;
                if (vec_ok && gr + 3 < r_end) {
                    const float4 x = *reinterpret_cast<const float4 *>(p);
                    v[0] = x.x; v[1] = x.y; v[2] = x.z; v[3] = x.w;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (gr + i < r_end) v[i] = p[i];
                }
            }
            *reinterpret_cast<float4 *>(&tile[k][rq]) = make_float4(v[0], v[1], v[2], v[3]);
        }
    }
}

template <bool A_K_CONTIG, bool B_K_CONTIG>
__global__ void __launch_bounds__(kThreads) gemm_kernel(const GemmArgs g, int a_vec_ok, int b_vec_ok) {
    __shared__ __attribute__((aligned(16))) float As[BK][BM + PAD];
    __shared__ __attribute__((aligned(16))) float Bs[BK][BN + PAD];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;  // this wavefront's quarter of the tile
    const int64_t m0 = int64_t(blockIdx.x) * BM, n0 = int64_t(blockIdx.y) * BN;
    const int64_t k_begin = int64_t(blockIdx.z) * g.k_per_split;
    const int64_t k_end = k_begin + g.k_per_split < g.K ? k_begin + g.k_per_split : g.K;

    float16v acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int l32 = lane & 31, lk = lane >> 5;
    for (int64_t k0 = k_begin; k0 < k_end; k0 += BK) {
        stage_tile<A_K_CONTIG>(As, g.A, g.sam, g.sak, m0, g.M, k0, k_end, a_vec_ok != 0);
        stage_tile<B_K_CONTIG>(Bs, g.B, g.sbn, g.sbk, n0, g.N, k0, k_end, b_vec_ok != 0);
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            // operand layout of the 32x32x2 instruction: lane l holds A[l % 32][l / 32] and B[l / 32][l % 32]
            const float a0 = As[kk + lk][wm + l32], a1 = As[kk + lk][wm + 32 + l32];
            const float b0 = Bs[kk + lk][wn + l32], b1 = Bs[kk + lk][wn + 32 + l32];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
        __syncthreads();
    }

    // result layout: register v of lane l is C[8 * (v / 4) + 4 * (l / 32) + v % 4][l % 32]
    float *out = g.C;
    if (g.n_split > 1) out += int64_t(blockIdx.z) * g.M * g.ldc;  // partial planes of M x ldc
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t n = n0 + wn + j * 32 + l32;
            if (n >= g.N) continue;
            const float bv = (g.bias && g.n_split == 1) ? g.bias[n] : 0.0f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t m = m0 + wm + i * 32 + 8 * (v / 4) + 4 * lk + (v % 4);
                if (m >= g.M) continue;
                float r = acc[i][j][v] + bv;
                if (g.relu && g.n_split == 1) r = r > 0.0f ? r : 0.0f;
                out[m * g.ldc + n] = r;
            }
        }
}

// C = act(sum over the partial planes + bias)
__global__ void __launch_bounds__(256) gemm_reduce_kernel(const float *__restrict__ part, int n_split, float *__restrict__ C,
                                                          int64_t ldc, int64_t M, int64_t N, const float *__restrict__ bias,
                                                          int relu) {
    const int64_t total = M * N;
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t t = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; t < total; t += stride) {
        const int64_t m = t / N, n = t - m * N;
        float s = 0.0f;
        for (int p = 0; p < n_split; ++p) s += part[(int64_t(p) * M + m) * N + n];
        if (bias) s += bias[n];
        if (relu) s = s > 0.0f ? s : 0.0f;
        C[m * ldc + n] = s;
    }
}

}  // namespace

// How many partial planes the reduction over k is split into.
static int64_t choose_split(int64_t M, int64_t N, int64_t K) {
    const int64_t tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
    if (tiles >= 512 || K < 4096) return 1;
    int64_t split = (1024 + tiles - 1) / tiles;           // aim at ~4 workgroups per compute unit
    const int64_t max_split = K / 1024 > 0 ? K / 1024 : 1;  // at least 1024 k-steps per split
    if (split > max_split) split = max_split;
    if (split > 4096) split = 4096;
    return split < 1 ? 1 : split;
}

extern "C" GNN_API int64_t gnn_matmul_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    const int64_t split = choose_split(M, N, K);
    return split > 1 ? split * M * N * int64_t(sizeof(float)) : 0;
}

extern "C" GNN_API int gnn_matmul(const float *A, int64_t lda, int trans_a, const float *B, int64_t ldb, int trans_b,
                                  float *C, int64_t ldc, int64_t M, int64_t N, int64_t K, const float *bias, int relu,
                                  void *workspace, int64_t workspace_bytes, void *stream_) {
    if (M < 0 || N < 0 || K < 0) return GNN_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return GNN_OK;
    if (!C || ldc < N) return GNN_ERR_INVALID_ARG;
    if (K > 0 && (!A || !B)) return GNN_ERR_INVALID_ARG;
    // stored shapes: A is [M, K] (or [K, M] when trans_a), B is [K, N] (or [N, K] when trans_b)
    if (K > 0 && (lda < (trans_a ? M : K) || ldb < (trans_b ? K : N))) return GNN_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(C) % 4 || reinterpret_cast<uintptr_t>(A) % 4 || reinterpret_cast<uintptr_t>(B) % 4)
        return GNN_ERR_INVALID_ARG;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    (void)hipGetLastError();

    GemmArgs g{};
    g.A = A; g.B = B; g.C = C; g.bias = bias;
    g.sam = trans_a ? 1 : lda;  g.sak = trans_a ? lda : 1;
    g.sbk = trans_b ? 1 : ldb;  g.sbn = trans_b ? ldb : 1;
    g.ldc = ldc; g.M = M; g.N = N; g.K = K;
    g.relu = relu ? 1 : 0;
    int64_t split = choose_split(M, N, K);
    if (split > 1 && (!workspace || workspace_bytes < split * M * N * int64_t(sizeof(float)))) split = 1;
    g.n_split = int32_t(split);
    g.k_per_split = split > 1 ? ((K + split - 1) / split + BK - 1) / BK * BK : (K > 0 ? K : 1);
    if (split > 1) {
        g.C = static_cast<float *>(workspace);
        g.ldc = N;
    }
    const int64_t gx = (M + BM - 1) / BM, gy = (N + BN - 1) / BN;
    if (gx > INT32_MAX || gy > 65535 || split > 65535) return GNN_ERR_UNSUPPORTED;
    dim3 grid(static_cast<unsigned>(gx), static_cast<unsigned>(gy), static_cast<unsigned>(split));
    const int a_vec = (lda % 4 == 0 && reinterpret_cast<uintptr_t>(A) % 16 == 0) ? 1 : 0;
    const int b_vec = (ldb % 4 == 0 && reinterpret_cast<uintptr_t>(B) % 16 == 0) ? 1 : 0;
    if (!trans_a && !trans_b) gemm_kernel<true, false><<<grid, kThreads, 0, stream>>>(g, a_vec, b_vec);
    else if (!trans_a && trans_b) gemm_kernel<true, true><<<grid, kThreads, 0, stream>>>(g, a_vec, b_vec);
    else if (trans_a && !trans_b) gemm_kernel<false, false><<<grid, kThreads, 0, stream>>>(g, a_vec, b_vec);
    else gemm_kernel<false, true><<<grid, kThreads, 0, stream>>>(g, a_vec, b_vec);
    if (hipGetLastError() != hipSuccess) return GNN_ERR_LAUNCH;
    if (split > 1) {
        int64_t blocks = (M * N + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        gemm_reduce_kernel<<<static_cast<unsigned>(blocks), 256, 0, stream>>>(static_cast<const float *>(workspace), int(split), C, ldc,
                                                                               M, N, bias, relu ? 1 : 0);
        if (hipGetLastError() != hipSuccess) return GNN_ERR_LAUNCH;
    }
    return GNN_OK;
}
