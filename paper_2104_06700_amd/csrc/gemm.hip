// Dense update of a GNN layer (the MLP step that follows the aggregation, Section 6.3 "Memory"):
//
//   C[m, n] = act( sum_k opA(A)[m, k] * opB(B)[k, n] + bias[n] )
//
// fp32 in, fp32 out, on the matrix cores: v_mfma_f32_32x32x2_f32 multiplies exact fp32 products and
// accumulates in fp32, so the result meets the same tolerance as the aggregation.  A workgroup of
// four wavefronts owns a 128 x 128 tile of C, each wavefront a 64 x 64 quarter as 2 x 2 MFMA
// tiles (256 x 64 or 256 x 32 tiles for narrow outputs).  A and B tiles of 16 k-steps are staged
// through LDS k-major ([k][m] and [k][n]), so that the 32 lanes of an MFMA operand read
// consecutive words; the global loads follow whichever direction of the operand is contiguous
// and are issued one tile ahead, so they fly while the matrix cores work on the current tile.  The
// reduction over a very long k (the weight gradient: k = number of vertices) is split into parts
// whose partial tiles a second kernel adds in order (deterministic, no atomics).
#include "common.h"

namespace {

constexpr int BK = 16;
constexpr int PAD = 4;  // row stride rows + PAD: k-rows start 4 banks apart
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
    gnn_packed_target packed;  // active: the result goes into a producer-side layout instead of C
    // Rectifier gate folded into the operand loads (the backward pass of a layer multiplies by
    // G = dH where H > 0): an element of A (of B) counts as 0 where the gate matrix, which has the
    // operand's shape and strides, is not positive.  colsum: [n_split][N] column sums of opB(B) after
    // its gate (the bias gradient), written by the workgroups of the first tile row.
    const float *a_gate, *b_gate;
    float *colsum;
    // Tile order.  The launch is one-dimensional and workgroup b runs on XCD b % 8, each with an L2 of its own.
    // The tiles that read the same rows of an operand (the column tiles of one row tile of a tall product; all
    // tiles of one part of a split reduction) get ids 8 apart: the same XCD, one after the other, so the second
    // read of those rows hits that XCD's L2.  inner = number of such tiles (0: plain order, x fastest).
    int32_t gx, gy, gz, inner;
};

// One [ROWS x BK] tile of an operand on its way from global memory to LDS (stored k-major as
// tile[k][r]).  X(r, k) = base[r * sr + k * sk].  K_CONTIG: sk == 1 (threads run along k), else
// sr == 1 (threads run along the rows); 16-byte loads when aligned.  load() and store() are
// separate so that the loads of the next tile are in flight while the matrix cores work.
template <bool K_CONTIG, int ROWS, bool GATED = false>
struct Stager {
    static constexpr int QUADS = ROWS * BK / 4;
    static constexpr int PER_THREAD = (QUADS + kThreads - 1) / kThreads;
    float v[PER_THREAD][4];
    float gate[GATED ? PER_THREAD : 1][4];  // the gate's elements travel beside the operand's and are applied in store()

    // Whole tiles of an aligned operand: the thread keeps the address of its quad 0 in the tile at k_begin; quad h
    // lies a uniform step further, a later tile a uniform offset further; rows are checked against a 32-bit
    // count.  The kernel's main loop uses only this path, so that it stays a few hundred instructions long: with
    // the general path below inlined (64-bit address arithmetic and a check per element, for every quad of up to
    // three matrices) the loop of the gated products outgrew what the instruction cache serves at full speed.
    const float *p0;
    int64_t step_h, k_step, gate_off;
    int32_t rows_left;

    __device__ __forceinline__ void init(const float *__restrict__ base, const float *__restrict__ gate_base, int64_t sr, int64_t sk,
                                         int64_t r0, int64_t r_end, int64_t k_begin) {
        const int q = int(threadIdx.x);
        if (K_CONTIG) {
            p0 = base + (r0 + (q >> 2)) * sr + k_begin + (q & 3) * 4;
            step_h = (kThreads / 4) * sr;
            k_step = 1;
        } else {
            p0 = base + (k_begin + q / (ROWS / 4)) * sk + r0 + (q % (ROWS / 4)) * 4;
            step_h = (kThreads / (ROWS / 4)) * sk;
            k_step = sk;
        }
        gate_off = (GATED && gate_base) ? gate_base - base : 0;
        const int64_t left = r_end - r0;
        rows_left = left > 0x7fffffff ? 0x7fffffff : int32_t(left);
    }

    // k_off = first k of the tile - k_begin (uniform); the tile lies inside the k range whole
    __device__ __forceinline__ void load_whole_tile(int64_t k_off, bool gated) {
        const float *pt = p0 + k_off * k_step;
#pragma unroll
        for (int h = 0; h < PER_THREAD; ++h) {
            const int q = int(threadIdx.x) + h * kThreads;
            if (QUADS % kThreads != 0 && q >= QUADS) continue;
            const int first_row = K_CONTIG ? (q >> 2) : (q % (ROWS / 4)) * 4;
            const int rows = K_CONTIG ? 1 : 4;  // rows this quad touches
            const float *p = pt + h * step_h;
            if (first_row + rows <= rows_left) {
                const float4 x = *reinterpret_cast<const float4 *>(p);
                v[h][0] = x.x; v[h][1] = x.y; v[h][2] = x.z; v[h][3] = x.w;
                if constexpr (GATED) {
                    if (gated) {
                        const float4 y = *reinterpret_cast<const float4 *>(p + gate_off);
                        gate[h][0] = y.x; gate[h][1] = y.y; gate[h][2] = y.z; gate[h][3] = y.w;
                    }
                }
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const bool ok = !K_CONTIG && first_row + i < rows_left;  // a quad of rows that straddles the end
                    v[h][i] = ok ? p[i] : 0.0f;
                    if constexpr (GATED) gate[h][i] = (ok && gated) ? p[gate_off + i] : 0.0f;
                }
            }
        }
    }

    __device__ __forceinline__ void load(const float *__restrict__ base, const float *__restrict__ gate_base, int64_t sr, int64_t sk,
                                         int64_t r0, int64_t r_end, int64_t k0, int64_t k_end, bool vec_ok) {
        fetch(base, v, sr, sk, r0, r_end, k0, k_end, vec_ok);
        if constexpr (GATED) {
            if (gate_base) fetch(gate_base, gate, sr, sk, r0, r_end, k0, k_end, vec_ok);
        }
    }

    template <int ROWS_OF_V>
    __device__ __forceinline__ void fetch(const float *__restrict__ base, float (&v)[ROWS_OF_V][4], int64_t sr, int64_t sk, int64_t r0,
                                          int64_t r_end, int64_t k0, int64_t k_end, bool vec_ok) {
#pragma unroll
        for (int h = 0; h < PER_THREAD; ++h) {
            const int q = int(threadIdx.x) + h * kThreads;
#pragma unroll
            for (int i = 0; i < 4; ++i) v[h][i] = 0.0f;
            if (QUADS % kThreads != 0 && q >= QUADS) continue;
            if (K_CONTIG) {
                const int r = q >> 2, kq = (q & 3) * 4;
                const int64_t gr = r0 + r, gk = k0 + kq;
                if (gr < r_end) {
                    const float *p = base + gr * sr + gk;
                    if (vec_ok && gk + 3 < k_end) {
                        const float4 x = *reinterpret_cast<const float4 *>(p);
                        v[h][0] = x.x; v[h][1] = x.y; v[h][2] = x.z; v[h][3] = x.w;
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (gk + i < k_end) v[h][i] = p[i];
                    }
                }
            } else {
                const int k = q / (ROWS / 4), rq = (q % (ROWS / 4)) * 4;
                const int64_t gk = k0 + k, gr = r0 + rq;
                if (gk < k_end) {
                    const float *p = base + gk * sk + gr;
                    if (vec_ok && gr + 3 < r_end) {
                        const float4 x = *reinterpret_cast<const float4 *>(p);
                        v[h][0] = x.x; v[h][1] = x.y; v[h][2] = x.z; v[h][3] = x.w;
                    } else {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (gr + i < r_end) v[h][i] = p[i];
                    }
                }
            }
        }
    }

    // Adds what this thread staged (after store() applied the gate) to its sums over k: for an operand whose
    // rows are contiguous a thread holds the same four rows in every tile.
    __device__ __forceinline__ void add_to_row_sums(float (&acc)[4]) const {
        static_assert(!K_CONTIG, "row sums are kept for row-contiguous operands only");
#pragma unroll
        for (int h = 0; h < PER_THREAD; ++h) {
            if (QUADS % kThreads != 0 && int(threadIdx.x) + h * kThreads >= QUADS) continue;
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] += v[h][i];
        }
    }

    __device__ __forceinline__ void store(float (*tile)[ROWS + PAD], bool gated) {
        if constexpr (GATED) {
            if (gated) {
#pragma unroll
                for (int h = 0; h < PER_THREAD; ++h)
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[h][i] = gate[h][i] > 0.0f ? v[h][i] : 0.0f;
            }
        }
#pragma unroll
        for (int h = 0; h < PER_THREAD; ++h) {
            const int q = int(threadIdx.x) + h * kThreads;
            if (QUADS % kThreads != 0 && q >= QUADS) continue;
            if (K_CONTIG) {
                const int r = q >> 2, kq = (q & 3) * 4;
#pragma unroll
                for (int i = 0; i < 4; ++i) tile[kq + i][r] = v[h][i];
            } else {
                const int k = q / (ROWS / 4), rq = (q % (ROWS / 4)) * 4;
                *reinterpret_cast<float4 *>(&tile[k][rq]) = make_float4(v[h][0], v[h][1], v[h][2], v[h][3]);
            }
        }
    }
};

// Workgroup tile (WM * TI * 32) x (WN * TJ * 32): WM x WN wavefronts, each TI x TJ MFMA tiles.
// FOLD: 0 = plain operands; 1 = A may carry a gate; 2 = B may carry a gate and its column sums may be asked for.
// (The 256 x 64 tile with a gated operand stages 32 more registers: three waves per SIMD instead of spilling.)
template <bool A_K_CONTIG, bool B_K_CONTIG, int WM, int WN, int TI, int TJ, int FOLD = 0>
__global__ void __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu((FOLD != 0 && WM == 4 && TJ == 2) ? 3 : 4, 8))) gemm_kernel(const GemmArgs g, int a_vec_ok, int b_vec_ok) {
    static_assert(WM * WN == kThreads / 64, "four wavefronts");
    constexpr int BM = WM * TI * 32, BN = WN * TJ * 32;
    __shared__ __attribute__((aligned(16))) float As[BK][BM + PAD];
    __shared__ __attribute__((aligned(16))) float Bs[BK][BN + PAD];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int wm = (wave / WN) * TI * 32, wn = (wave % WN) * TJ * 32;  // this wavefront's part of the tile
    int64_t bx, by, bz;
    {
        const int64_t b = blockIdx.x;
        if (g.inner > 0) {
            const int64_t per = int64_t(8) * g.inner, r = b % per;
            const int64_t outer = b / per * 8 + (r & 7), in = r >> 3;
            if (g.gz > 1) { bz = outer; bx = in % g.gx; by = in / g.gx; }
            else { bx = outer; by = in; bz = 0; }
            if (bx >= g.gx || bz >= g.gz) return;  // the last group of 8 may be incomplete (whole workgroup leaves)
        } else {
            bx = b % g.gx;
            by = b / g.gx % g.gy;
            bz = b / (int64_t(g.gx) * g.gy);
        }
    }
    const int64_t m0 = bx * BM, n0 = by * BN;
    const int64_t k_begin = bz * g.k_per_split;
    const int64_t k_end = k_begin + g.k_per_split < g.K ? k_begin + g.k_per_split : g.K;

    float16v acc[TI][TJ];
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    Stager<A_K_CONTIG, BM, FOLD == 1> sa;
    Stager<B_K_CONTIG, BN, FOLD == 2> sb;
    const bool a_gated = FOLD == 1 && g.a_gate, b_gated = FOLD == 2 && g.b_gate;
    const bool sums = FOLD == 2 && g.colsum && bx == 0;  // the first tile row also adds up the columns of B (uniform)
    float col_sum[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    const int l32 = lane & 31, lk = lane >> 5;
    auto stage = [&]() {  // registers -> LDS
        sa.store(As, a_gated);
        sb.store(Bs, b_gated);
        if constexpr (FOLD == 2) {
            if (sums) sb.add_to_row_sums(col_sum);  // rows past k_end were staged as zeros
        }
    };
    auto multiply = [&]() {
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            // operand layout of the 32x32x2 instruction: lane l holds A[l % 32][l / 32] and B[l / 32][l % 32]
            float a[TI], b[TJ];
#pragma unroll
            for (int i = 0; i < TI; ++i) a[i] = As[kk + lk][wm + i * 32 + l32];
#pragma unroll
            for (int j = 0; j < TJ; ++j) b[j] = Bs[kk + lk][wn + j * 32 + l32];
#pragma unroll
            for (int i = 0; i < TI; ++i)
#pragma unroll
                for (int j = 0; j < TJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
    };
    auto load_any = [&](int64_t k0) {
        sa.load(g.A, g.a_gate, g.sam, g.sak, m0, g.M, k0, k_end, a_vec_ok != 0);
        sb.load(g.B, g.b_gate, g.sbn, g.sbk, n0, g.N, k0, k_end, b_vec_ok != 0);
    };
    // Tiles t = 0 .. n_tiles - 1; the first n_fast of them are whole tiles of aligned operands.  The loads of tile
    // t + 1 are issued before tile t is multiplied, so they fly while the matrix cores work.
    const int64_t n_tiles = k_begin < k_end ? (k_end - k_begin + BK - 1) / BK : 0;
    const int64_t n_fast = (a_vec_ok && b_vec_ok && k_begin < k_end) ? (k_end - k_begin) / BK : 0;
    sa.init(g.A, g.a_gate, g.sam, g.sak, m0, g.M, k_begin);
    sb.init(g.B, g.b_gate, g.sbn, g.sbk, n0, g.N, k_begin);
    if (n_fast > 0) {
        sa.load_whole_tile(0, a_gated);
        sb.load_whole_tile(0, b_gated);
    } else if (n_tiles > 0) {
        load_any(k_begin);
    }
    int64_t t = 0;
    for (; t + 1 < n_fast; ++t) {  // the main loop: tile t + 1 is a whole one
        stage();
        __syncthreads();
        sa.load_whole_tile((t + 1) * BK, a_gated);
        sb.load_whole_tile((t + 1) * BK, b_gated);
        multiply();
        __syncthreads();
    }
    for (; t < n_tiles; ++t) {  // what is left: a last partial tile, or every tile of an operand that is not aligned
        stage();
        __syncthreads();
        if (t + 1 < n_tiles) load_any(k_begin + (t + 1) * BK);
        multiply();
        __syncthreads();
    }

    if constexpr (FOLD == 2) {
        if (sums) {
            // a thread holds 4 columns of one k-row of every tile; the threads that hold the same columns are
            // added in thread order through LDS (the operand tiles are no longer needed)
            constexpr int GROUPS = BN / 4, SLOTS = kThreads / GROUPS;
            float *scr = &As[0][0];
            static_assert(SLOTS * BN <= BK * (BM + PAD), "scratch fits the A tile");
            const int grp = int(threadIdx.x) % GROUPS, slot = int(threadIdx.x) / GROUPS;
#pragma unroll
            for (int i = 0; i < 4; ++i) scr[slot * BN + grp * 4 + i] = col_sum[i];
            __syncthreads();
            if (int(threadIdx.x) < BN && n0 + int(threadIdx.x) < g.N) {
                float tsum = 0.0f;
                for (int sl = 0; sl < SLOTS; ++sl) tsum += scr[sl * BN + threadIdx.x];
                g.colsum[bz * g.N + n0 + threadIdx.x] = tsum;
            }
        }
    }

    // result layout: register v of lane l is C[8 * (v / 4) + 4 * (l / 32) + v % 4][l % 32]
    float *out = g.C;
    if (g.n_split > 1) out += bz * g.M * g.ldc;  // partial planes of M x ldc
    const gnn_packed_target &pk = g.packed;
    if (pk.active) {
        // producer-side layout: the 32 lanes of a row write one 128-byte line of a slice table (or a piece of the
        // tail) at the row's rank; rank and factor of a row are looked up once for all its column tiles
        float *pk_col[TJ];
        int64_t pk_ld[TJ];
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
            const int64_t n = n0 + wn + j * 32 + l32;
            pk_col[j] = nullptr;
            pk_ld[j] = 0;
            if (n < g.N) {
                if (n < pk.main_cols) { pk_col[j] = pk.base + (n >> 5) * pk.table_stride + (n & 31); pk_ld[j] = 32; }
                else { pk_col[j] = pk.tail + (n - pk.main_cols); pk_ld[j] = pk.tail_ld; }
            }
        }
#pragma unroll
        for (int i = 0; i < TI; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t m = m0 + wm + i * 32 + 8 * (v / 4) + 4 * lk + (v % 4);
                if (m >= g.M) continue;
                const int64_t row = pk.rank[m];
                const float fac = gnn_row_factor(pk.scale_mode, pk.scale_mode ? pk.counts[m] : 0);
#pragma unroll
                for (int j = 0; j < TJ; ++j)
                    if (pk_col[j]) pk_col[j][row * pk_ld[j]] = acc[i][j][v] * fac;
            }
        return;
    }
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < TJ; ++j) {
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

template <int WM, int WN, int TI, int TJ>
void launch_gemm(bool a_k, bool b_k, dim3 grid, hipStream_t stream, const GemmArgs &g, int a_vec, int b_vec) {
    // the two products of a layer's backward pass that take G = (dH where H > 0) as an operand
    if (g.a_gate && b_k) gemm_kernel<true, true, WM, WN, TI, TJ, 1><<<grid, kThreads, 0, stream>>>(g, a_vec, b_vec);
    else if (g.a_gate) gemm_kernel<true, false, WM, WN, TI, TJ, 1><<<grid, kThreads, 0, stream>>>(g, a_vec, b_vec);
    else if (g.b_gate || g.colsum) gemm_kernel<false, false, WM, WN, TI, TJ, 2><<<grid, kThreads, 0, stream>>>(g, a_vec, b_vec);
    else if (a_k && !b_k) gemm_kernel<true, false, WM, WN, TI, TJ><<<grid, kThreads, 0, stream>>>(g, a_vec, b_vec);
    else if (a_k && b_k) gemm_kernel<true, true, WM, WN, TI, TJ><<<grid, kThreads, 0, stream>>>(g, a_vec, b_vec);
    else if (!a_k && !b_k) gemm_kernel<false, false, WM, WN, TI, TJ><<<grid, kThreads, 0, stream>>>(g, a_vec, b_vec);
    else gemm_kernel<false, true, WM, WN, TI, TJ><<<grid, kThreads, 0, stream>>>(g, a_vec, b_vec);
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
// Tile width: 128 columns, or 64 / 32 (with 256 rows) for narrow outputs such as class scores.
static void choose_tile(int64_t N, int64_t *bm, int64_t *bn) {
    if (N > 64) { *bm = 128; *bn = 128; }
    else if (N > 32) { *bm = 256; *bn = 64; }
    else { *bm = 256; *bn = 32; }
}

static int64_t choose_split(int64_t M, int64_t N, int64_t K) {
    int64_t BM, BN;
    choose_tile(N, &BM, &BN);
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
                                  void *workspace, int64_t workspace_bytes, void *stream) {
    return gnn_matmul_impl(A, lda, trans_a, B, ldb, trans_b, C, ldc, M, N, K, bias, relu, workspace, workspace_bytes,
                           static_cast<hipStream_t>(stream));
}

int gnn_matmul_impl(const float *A, int64_t lda, int trans_a, const float *B, int64_t ldb, int trans_b, float *C, int64_t ldc,
                    int64_t M, int64_t N, int64_t K, const float *bias, int relu, void *workspace, int64_t workspace_bytes,
                    hipStream_t stream, const gnn_packed_target *packed, gnn_gemm_fold *fold) {
    if (M < 0 || N < 0 || K < 0) return GNN_ERR_INVALID_ARG;
    if (fold) fold->n_planes = 0;
    if (M == 0 || N == 0) return GNN_OK;
    const bool to_packed = packed && packed->active;
    if (!to_packed && (!C || ldc < N)) return GNN_ERR_INVALID_ARG;
    if (K > 0 && (!A || !B)) return GNN_ERR_INVALID_ARG;
    // stored shapes: A is [M, K] (or [K, M] when trans_a), B is [K, N] (or [N, K] when trans_b)
    if (K > 0 && (lda < (trans_a ? M : K) || ldb < (trans_b ? K : N))) return GNN_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(C) % 4 || reinterpret_cast<uintptr_t>(A) % 4 || reinterpret_cast<uintptr_t>(B) % 4)
        return GNN_ERR_INVALID_ARG;
    if (to_packed && (bias || relu)) return GNN_ERR_UNSUPPORTED;  // the aggregation that follows applies them
    if (to_packed && (!packed->base || !packed->rank || (packed->scale_mode && !packed->counts) ||
                      (packed->main_cols < N && !packed->tail)))
        return GNN_ERR_INVALID_ARG;
    // gates and column sums exist for the operand layouts of the layer's backward products only
    if (fold && fold->a_gate && (trans_a || fold->b_gate || fold->colsum)) return GNN_ERR_UNSUPPORTED;
    if (fold && (fold->b_gate || fold->colsum) && (!trans_a || trans_b)) return GNN_ERR_UNSUPPORTED;
    (void)hipGetLastError();

    GemmArgs g{};
    g.A = A; g.B = B; g.C = C; g.bias = bias;
    if (fold) { g.a_gate = fold->a_gate; g.b_gate = fold->b_gate; g.colsum = fold->colsum; }
    g.sam = trans_a ? 1 : lda;  g.sak = trans_a ? lda : 1;
    g.sbk = trans_b ? 1 : ldb;  g.sbn = trans_b ? ldb : 1;
    g.ldc = ldc; g.M = M; g.N = N; g.K = K;
    g.relu = relu ? 1 : 0;
    int64_t split = choose_split(M, N, K);
    if (split > 1 && (!workspace || workspace_bytes < split * M * N * int64_t(sizeof(float)))) split = 1;
    if (to_packed) {  // tall results only: no split reduction on this route
        split = 1;
        g.packed = *packed;
    }
    if (fold && fold->colsum) {
        if (fold->colsum_planes < split) return GNN_ERR_INVALID_ARG;
        fold->n_planes = split;
    }
    g.n_split = int32_t(split);
    g.k_per_split = split > 1 ? ((K + split - 1) / split + BK - 1) / BK * BK : (K > 0 ? K : 1);
    if (split > 1) {
        g.C = static_cast<float *>(workspace);
        g.ldc = N;
    }
    int64_t BM, BN;
    choose_tile(N, &BM, &BN);
    const int64_t gx = (M + BM - 1) / BM, gy = (N + BN - 1) / BN;
    if (gx > INT32_MAX || gy > 65535 || split > 65535) return GNN_ERR_UNSUPPORTED;
    g.gx = int32_t(gx); g.gy = int32_t(gy); g.gz = int32_t(split);
    int64_t n_groups = gx * gy * split;
    const int64_t inner = split > 1 ? gx * gy : gy, outer = split > 1 ? split : gx;
    if (inner >= 2 && inner <= 16 && outer >= 16) {
        g.inner = int32_t(inner);
        n_groups = (outer + 7) / 8 * 8 * inner;
    }
    if (n_groups > INT32_MAX) return GNN_ERR_UNSUPPORTED;
    dim3 grid(static_cast<unsigned>(n_groups));
    const int a_vec = (lda % 4 == 0 && reinterpret_cast<uintptr_t>(A) % 16 == 0 && reinterpret_cast<uintptr_t>(g.a_gate) % 16 == 0) ? 1 : 0;
    const int b_vec = (ldb % 4 == 0 && reinterpret_cast<uintptr_t>(B) % 16 == 0 && reinterpret_cast<uintptr_t>(g.b_gate) % 16 == 0) ? 1 : 0;
    const bool a_k = !trans_a, b_k = trans_b != 0;  // is k the contiguous direction of the operand?
    if (BN == 128) launch_gemm<2, 2, 2, 2>(a_k, b_k, grid, stream, g, a_vec, b_vec);
    else if (BN == 64) launch_gemm<4, 1, 2, 2>(a_k, b_k, grid, stream, g, a_vec, b_vec);
    else launch_gemm<4, 1, 2, 1>(a_k, b_k, grid, stream, g, a_vec, b_vec);
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
