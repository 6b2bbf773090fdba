// General aggregation primitive (Section 4.1, Algorithm 1) with the operator table of Table 1:
//
//   f_O[v, j] = reduce_{e = (u -> v) in row v}  binop(f_V[u, j], f_E[e, j])
//
// and its gradients.  Same execution scheme as the sum-only kernels of aggregate.hip -- row
// groups of G lanes (C column lanes x SR edge slots) chosen per degree bin, coalesced index tiles
// handed out by cross-lane shuffles, register accumulation, one owner per output row, hub rows cut
// into pieces that a second kernel combines in order -- with the message and the reduction as
// template parameters.  max / min carry the winning edge position beside the value and combine
// (value, position) pairs lexicographically, so the winner is the lowest position among equals
// whatever the slot layout.  fp32 only; 16-byte or 4-byte accesses.
#include "common.h"

#include <math.h>

namespace {

constexpr int kBlockThreads = 256;
constexpr int kWavesPerBlock = kBlockThreads / 64;

constexpr int kKindHubPieces = GNN_BIN_HUB_PIECES;
using ApBin = gnn_bin_desc;

struct ApArgs {
    const void *indptr;
    const int32_t *indices;
    const int64_t *eid;
    const float *fV;   // gathered vertex operand (forward: f_V; edge gradient: f_V)
    const float *fE;   // edge operand
    const float *dO;   // edge gradient only: gradient of the output rows
    float *out;        // forward: f_O; edge gradient: dfE
    int32_t *arg_out;  // forward, max / min: winning positions (or nullptr)
    int64_t ld_arg;    // row stride of arg_out (d, or the padded width of a staged call)
    const int32_t *arg_in;  // edge gradient, max / min
    int64_t ldv, lde, ldo;
    int32_t d;
    int32_t ip64;
    const int32_t *row_perm;
    const int64_t *chunks;
    float *pval;       // hub pieces: partial values   [n_chunks, ldp]
    int32_t *parg;     // hub pieces: partial winners  [n_chunks, ldp]
    int64_t ldp;
    int32_t n_bins;
    int32_t slab_cols;    // columns one workgroup covers
    int32_t col0;         // first column of this launch
    int32_t col_end;      // one past its last column
    int32_t log2_slices;  // > 0: workgroup b serves column slab (b % n_slices) of the launch, so that an
                          // XCD (workgroups go to the 8 XCDs round-robin) keeps gathering the same lines
                          // of every row; 0: the slab is blockIdx.y
    ApBin bins[GNN_MAX_BINS + 1];
};

__device__ __forceinline__ int64_t load_ip(const void *indptr, int ip64, int64_t i) {
    return ip64 ? static_cast<const int64_t *>(indptr)[i]
                : static_cast<int64_t>(static_cast<const int32_t *>(indptr)[i]);
}

template <int VEC> __device__ __forceinline__ void load_f(const float *p, float (&v)[VEC]) {
    if constexpr (VEC == 4) {
        const float4 t = *reinterpret_cast<const float4 *>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        v[0] = *p;
    }
}
typedef float f32x4 __attribute__((ext_vector_type(4)));
// non-temporal variant for rows of rarely gathered ("cold") sources
template <int VEC> __device__ __forceinline__ void load_f_nt(const float *p, float (&v)[VEC]) {
    if constexpr (VEC == 4) {
        const f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        v[0] = __builtin_nontemporal_load(p);
    }
}
template <int VEC> __device__ __forceinline__ void store_f(float *p, const float (&v)[VEC]) {
    if constexpr (VEC == 4) *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    else *p = v[0];
}
template <int VEC> __device__ __forceinline__ void load_i(const int32_t *p, int32_t (&v)[VEC]) {
    if constexpr (VEC == 4) {
        const int4 t = *reinterpret_cast<const int4 *>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        v[0] = *p;
    }
}
template <int VEC> __device__ __forceinline__ void store_i(int32_t *p, const int32_t (&v)[VEC]) {
    if constexpr (VEC == 4) *reinterpret_cast<int4 *>(p) = make_int4(v[0], v[1], v[2], v[3]);
    else *p = v[0];
}

__device__ __forceinline__ int64_t shfl_i64(int64_t v, int src_lane) {
    const int lo = __shfl(int(uint32_t(uint64_t(v))), src_lane);
    const int hi = __shfl(int(uint32_t(uint64_t(v) >> 32)), src_lane);
    return int64_t((uint64_t(uint32_t(hi)) << 32) | uint64_t(uint32_t(lo)));
}

// One correctly rounded fp32 operation per message (max / min compare these values with the
// oracle's bit for bit, so nothing may be fused into them).
template <int BIN> __device__ __forceinline__ float message(float x, float y) {
    if constexpr (BIN == GNN_BIN_ADD) return __fadd_rn(x, y);
    else if constexpr (BIN == GNN_BIN_SUB) return __fsub_rn(x, y);
    else if constexpr (BIN == GNN_BIN_MUL) return __fmul_rn(x, y);
    else if constexpr (BIN == GNN_BIN_DIV) return __fdiv_rn(x, y);
    else if constexpr (BIN == GNN_BIN_COPY_LHS) return x;
    else return y;
}

template <int RED> __device__ __forceinline__ bool better(float cand, float best) {
    return RED == GNN_RED_MAX ? cand > best : cand < best;
}

// Which bin a workgroup serves, and the row (or hub piece) and edge range its group owns.
struct Group {
    int G, SR, C, log2_c, lane_in_g, gbase, s, c;
    int64_t row, e0, e1, piece;
    bool is_piece;
};

__device__ __forceinline__ Group locate_group(const ApArgs &a, int64_t vblock) {
    Group g;
    const int lane = threadIdx.x & 63;
    const int wave_in_block = threadIdx.x >> 6;
    int b = 0;
    for (int i = 1; i < a.n_bins; ++i)
        if (vblock >= a.bins[i].first_block) b = i;
    const ApBin bin = a.bins[b];
    const int64_t wave_in_bin = (vblock - bin.first_block) * kWavesPerBlock + wave_in_block;
    g.G = 1 << bin.log2_g;
    g.SR = 1 << bin.log2_sr;
    g.log2_c = bin.log2_g - bin.log2_sr;
    g.C = 1 << g.log2_c;
    g.lane_in_g = lane & (g.G - 1);
    g.gbase = lane - g.lane_in_g;
    g.s = g.lane_in_g >> g.log2_c;
    g.c = g.lane_in_g & (g.C - 1);
    g.row = -1;
    g.e0 = g.e1 = 0;
    g.piece = -1;
    g.is_piece = bin.kind == kKindHubPieces;
    if (g.is_piece) {
        if (wave_in_bin < bin.n_items) {
            const int64_t *p = a.chunks + 3 * (bin.item_begin + wave_in_bin);
            g.row = p[0]; g.e0 = p[1]; g.e1 = p[2];
            g.piece = bin.item_begin + wave_in_bin;
        }
    } else {
        const int64_t item = wave_in_bin * (64 >> bin.log2_g) + (lane >> bin.log2_g);
        if (item < bin.n_items) {
            g.row = a.row_perm ? int64_t(a.row_perm[bin.item_begin + item]) : bin.item_begin + item;
            g.e0 = load_ip(a.indptr, a.ip64, g.row);
            g.e1 = load_ip(a.indptr, a.ip64, g.row + 1);
        }
    }
    return g;
}

// ------------------------------------------------------------------ forward
// EWIDE: f_E has one column per feature column (else one scalar per edge).
template <int BIN, int RED, int VEC, bool EWIDE>
__global__ void __launch_bounds__(kBlockThreads) ap_fwd_kernel(const ApArgs a) {
    constexpr bool USE_V = BIN != GNN_BIN_COPY_RHS;
    constexpr bool USE_E = BIN != GNN_BIN_COPY_LHS;
    constexpr bool WIDE = USE_E && EWIDE;
    constexpr int U = (VEC == 4 && (WIDE || RED != GNN_RED_SUM)) ? 4 : 8;  // edges in flight per slot (fewer where values and winners fill the registers)
    const int slab = a.log2_slices > 0 ? int(blockIdx.x) & ((1 << a.log2_slices) - 1) : int(blockIdx.y);
    const Group g = locate_group(a, int64_t(blockIdx.x) >> a.log2_slices);
    const int G = g.G, SR = g.SR;
    const int col = a.col0 + slab * a.slab_cols + g.c * VEC;
    const bool col_ok = col < a.col_end && g.c * VEC < a.slab_cols;
    const int64_t e0 = g.e0, e1 = g.e1;

    float acc[VEC];
    int32_t win[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        acc[i] = RED == GNN_RED_SUM ? 0.0f : (RED == GNN_RED_MAX ? -INFINITY : INFINITY);
        win[i] = -1;
    }

    auto fetch_tile = [&](int64_t e, int &u_out, float &y_out, int64_t &r_out) {
        u_out = 0; y_out = 1.0f; r_out = 0;
        if (e < e1) {
            u_out = a.indices[e];
            if (USE_E) {
                r_out = a.eid ? a.eid[e] : e;
                if (!EWIDE) y_out = a.fE[r_out * a.lde];
            }
        }
    };
    int nxt_u; float nxt_y; int64_t nxt_r;
    fetch_tile(e0 + g.lane_in_g, nxt_u, nxt_y, nxt_r);
    for (int64_t tile = e0; __any(tile < e1); tile += G) {
        const int my_u = nxt_u;
        const float my_y = nxt_y;
        const int64_t my_r = nxt_r;
        fetch_tile(tile + G + g.lane_in_g, nxt_u, nxt_y, nxt_r);
        const int64_t left = e1 - tile;
        const int n_tile = left < G ? (left > 0 ? int(left) : 0) : G;
        for (int j0 = 0; __any(j0 < n_tile); j0 += SR * U) {
            int u[U];
            float ys[U];
            int64_t r[U];
            bool ok[U];
#pragma unroll
            for (int k = 0; k < U; ++k) {
                const int j = j0 + k * SR + g.s;
                const int src_lane = g.gbase + (j & (G - 1));
                u[k] = __shfl(my_u, src_lane);
                ys[k] = (USE_E && !EWIDE) ? __shfl(my_y, src_lane) : 1.0f;
                r[k] = 0;
                if (WIDE) r[k] = a.eid ? shfl_i64(my_r, src_lane) : tile + j;
                ok[k] = j < n_tile && col_ok;
            }
            float x[U][VEC], y[U][VEC];
#pragma unroll
            for (int k = 0; k < U; ++k) {
#pragma unroll
                for (int i = 0; i < VEC; ++i) { x[k][i] = 0.0f; y[k][i] = ys[k]; }
                if (ok[k]) {
                    if (USE_V) {  // bit 31 of an index flags a cold source (plan-owned index copy, see aggregate.hip)
                        const float *xr = a.fV + int64_t(u[k] & 0x7FFFFFFF) * a.ldv + col;
                        if (u[k] < 0) load_f_nt<VEC>(xr, x[k]);
                        else load_f<VEC>(xr, x[k]);
                    }
                    if (WIDE) load_f<VEC>(a.fE + r[k] * a.lde + col, y[k]);
                } else {
#pragma unroll
                    for (int i = 0; i < VEC; ++i) y[k][i] = 1.0f;
                }
            }
#pragma unroll
            for (int k = 0; k < U; ++k) {
                const int32_t pos = int32_t(tile + j0 + k * SR + g.s);
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    if constexpr (RED == GNN_RED_SUM) {
                        float m;
                        if constexpr (BIN == GNN_BIN_ADD) m = x[k][i] + y[k][i];
                        else if constexpr (BIN == GNN_BIN_SUB) m = x[k][i] - y[k][i];
                        else if constexpr (BIN == GNN_BIN_MUL) m = x[k][i] * y[k][i];
                        else m = message<BIN>(x[k][i], y[k][i]);
                        acc[i] += ok[k] ? m : 0.0f;
                    } else {
                        const float m = message<BIN>(x[k][i], y[k][i]);
                        if (ok[k] && (win[i] < 0 || better<RED>(m, acc[i]))) { acc[i] = m; win[i] = pos; }
                    }
                }
            }
        }
    }

    // combine the edge slots of the group
    for (int off = g.C; off < G; off <<= 1) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            const float om = __shfl_xor(acc[i], off);
            if constexpr (RED == GNN_RED_SUM) {
                acc[i] += om;
            } else {
                const int32_t ow = __shfl_xor(win[i], off);
                const bool take = ow >= 0 && (win[i] < 0 || better<RED>(om, acc[i]) || (om == acc[i] && ow < win[i]));
                if (take) { acc[i] = om; win[i] = ow; }
            }
        }
    }

    if (g.row < 0 || g.s != 0 || !col_ok) return;
    if (g.is_piece) {
        store_f<VEC>(a.pval + g.piece * a.ldp + col, acc);
        if (RED != GNN_RED_SUM) store_i<VEC>(a.parg + g.piece * a.ldp + col, win);
        return;
    }
    if (RED != GNN_RED_SUM) {
#pragma unroll
        for (int i = 0; i < VEC; ++i)
            if (win[i] < 0) acc[i] = 0.0f;  // row without edges
        if (a.arg_out) store_i<VEC>(a.arg_out + g.row * a.ld_arg + col, win);
    }
    store_f<VEC>(a.out + g.row * a.ldo + col, acc);
}

// Combines the pieces of each hub row in ascending edge order and writes the row.
template <int RED>
__global__ void __launch_bounds__(256) ap_hub_finalize_kernel(const int32_t *__restrict__ hub_rows, int64_t n_hub,
                                                              const int64_t *__restrict__ piece_offsets,
                                                              const float *__restrict__ pval, const int32_t *__restrict__ parg,
                                                              int64_t ldp, float *__restrict__ out, int64_t ldo,
                                                              int32_t *__restrict__ arg_out, int64_t ld_arg, int d) {
    const int64_t i = blockIdx.x;
    if (i >= n_hub) return;
    const int64_t row = hub_rows[i];
    const int64_t p0 = piece_offsets[i], p1 = piece_offsets[i + 1];
    for (int col = threadIdx.x; col < d; col += blockDim.x) {
        float best = 0.0f;
        int32_t won = -1;
        for (int64_t p = p0; p < p1; ++p) {
            const float v = pval[p * ldp + col];
            if (RED == GNN_RED_SUM) {
                best += v;
            } else {
                const int32_t w = parg[p * ldp + col];
                if (w >= 0 && (won < 0 || better<RED>(v, best))) { best = v; won = w; }
            }
        }
        out[row * ldo + col] = best;
        if (RED != GNN_RED_SUM && arg_out) arg_out[row * ld_arg + col] = won;
    }
}

// ------------------------------------------------------------ edge gradient
// dfE[r(e), j] = dO[v, j] * d binop / dy, per edge of the forward graph; summed over j when the
// edge operand is a scalar.  MASKED: only where arg_in[v, j] == e (max / min).
template <int BIN, int VEC, bool EWIDE, bool MASKED>
__global__ void __launch_bounds__(kBlockThreads) ap_bwd_edge_kernel(const ApArgs a) {
    constexpr bool NEED_X = BIN == GNN_BIN_MUL || BIN == GNN_BIN_DIV;
    constexpr bool NEED_Y = BIN == GNN_BIN_DIV;
    constexpr int U = 4;
    const Group g = locate_group(a, blockIdx.x);
    const int G = g.G, SR = g.SR, C = g.C;
    const int64_t e0 = g.e0, e1 = g.e1;
    const int64_t row = g.row < 0 ? 0 : g.row;

    auto fetch_tile = [&](int64_t e, int &u_out, float &y_out, int64_t &r_out) {
        u_out = 0; y_out = 1.0f; r_out = 0;
        if (e < e1) {
            u_out = a.indices[e];
            r_out = a.eid ? a.eid[e] : e;
            if (NEED_Y && !EWIDE) y_out = a.fE[r_out * a.lde];
        }
    };
    int nxt_u; float nxt_y; int64_t nxt_r;
    fetch_tile(e0 + g.lane_in_g, nxt_u, nxt_y, nxt_r);
    for (int64_t tile = e0; __any(tile < e1); tile += G) {
        const int my_u = nxt_u;
        const float my_y = nxt_y;
        const int64_t my_r = nxt_r;
        fetch_tile(tile + G + g.lane_in_g, nxt_u, nxt_y, nxt_r);
        const int64_t left = e1 - tile;
        const int n_tile = left < G ? (left > 0 ? int(left) : 0) : G;
        for (int j0 = 0; __any(j0 < n_tile); j0 += SR * U) {
            int u[U];
            float ys[U];
            int64_t r[U];
            bool ok[U];
            float part[U];
#pragma unroll
            for (int k = 0; k < U; ++k) {
                const int j = j0 + k * SR + g.s;
                const int src_lane = g.gbase + (j & (G - 1));
                u[k] = __shfl(my_u, src_lane);
                ys[k] = (NEED_Y && !EWIDE) ? __shfl(my_y, src_lane) : 1.0f;
                r[k] = a.eid ? shfl_i64(my_r, src_lane) : tile + j;
                ok[k] = j < n_tile;
                part[k] = 0.0f;
            }
            for (int col = g.c * VEC; col < a.d; col += C * VEC) {
                float go[VEC];
                int32_t aw[VEC];
                load_f<VEC>(a.dO + row * a.ldo + col, go);
                if (MASKED) load_i<VEC>(a.arg_in + row * int64_t(a.d) + col, aw);
#pragma unroll
                for (int k = 0; k < U; ++k) {
                    if (!ok[k]) continue;
                    float x[VEC], y[VEC], gy[VEC];
#pragma unroll
                    for (int i = 0; i < VEC; ++i) { x[i] = 0.0f; y[i] = ys[k]; }
                    if (NEED_X) load_f<VEC>(a.fV + int64_t(u[k]) * a.ldv + col, x);
                    if (NEED_Y && EWIDE) load_f<VEC>(a.fE + r[k] * a.lde + col, y);
                    const int32_t pos = int32_t(tile + j0 + k * SR + g.s);
#pragma unroll
                    for (int i = 0; i < VEC; ++i) {
                        float t;
                        if constexpr (BIN == GNN_BIN_ADD || BIN == GNN_BIN_COPY_RHS) t = go[i];
                        else if constexpr (BIN == GNN_BIN_SUB) t = -go[i];
                        else if constexpr (BIN == GNN_BIN_MUL) t = go[i] * x[i];
                        else t = -go[i] * x[i] / (y[i] * y[i]);
                        if (MASKED && aw[i] != pos) t = 0.0f;
                        gy[i] = t;
                    }
                    if (EWIDE) {
                        store_f<VEC>(a.out + r[k] * a.lde + col, gy);
                    } else {
#pragma unroll
                        for (int i = 0; i < VEC; ++i) part[k] += gy[i];
                    }
                }
            }
            if (!EWIDE) {
#pragma unroll
                for (int k = 0; k < U; ++k) {
                    float t = part[k];
                    for (int off = 1; off < C; off <<= 1) t += __shfl_xor(t, off);
                    if (ok[k] && g.c == 0) a.out[r[k] * a.lde] = t;
                }
            }
        }
    }
}

// ------------------------------------------- vertex gradient of max / min
template <int BIN>
__global__ void __launch_bounds__(256) ap_scatter_arg_kernel(const int32_t *__restrict__ indices, const int64_t *__restrict__ eid,
                                                             const int32_t *__restrict__ arg, const float *__restrict__ dO,
                                                             int64_t ldo, const float *__restrict__ fE, int64_t lde, int ewide,
                                                             float *__restrict__ dfV, int64_t ldv, int64_t N, int d) {
    const int64_t total = N * d;
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t t = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; t < total; t += stride) {
        const int64_t v = t / d;
        const int j = int(t - v * d);
        const int32_t e = arg[t];
        if (e < 0) continue;
        float gx = dO[v * ldo + j];
        if (BIN == GNN_BIN_MUL || BIN == GNN_BIN_DIV) {
            const int64_t r = eid ? eid[e] : int64_t(e);
            const float y = fE[r * lde + (ewide ? j : 0)];
            gx = BIN == GNN_BIN_MUL ? gx * y : gx / y;
        }
        unsafeAtomicAdd(dfV + int64_t(indices[e]) * ldv + j, gx);
    }
}

__global__ void __launch_bounds__(256) fill_rows_kernel(float *__restrict__ p, int64_t ld, int64_t n_rows, int d, float value) {
    const int64_t total = n_rows * d;
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t t = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; t < total; t += stride) {
        const int64_t v = t / d;
        p[v * ld + (t - v * d)] = value;
    }
}

// ---------------------------------------------------------------- host side
bool aligned16(const void *p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }
bool aligned4(const void *p) { return reinterpret_cast<uintptr_t>(p) % 4 == 0; }

unsigned grid_1d(int64_t work, int64_t cap = int64_t(1) << 17) {
    int64_t b = (work + 255) / 256;
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return static_cast<unsigned>(b);
}

// Fills the bin table (heaviest work first) and returns the number of workgroups along x.
int64_t make_bins(ApArgs &a, const gnn_plan *plan, int64_t N, int log2_c) {
    if (plan) {
        a.row_perm = plan->row_perm;
        a.chunks = plan->chunks;
    }
    return gnn_fill_bins(a.bins, &a.n_bins, plan, N, log2_c);
}

struct Common {
    gnn_ap_opts o;
    int64_t ldv, lde, ldo;
    bool ewide;
    hipStream_t stream;
};

int check_common(const gnn_ap_opts *opts_in, int64_t N, int64_t d, int binop, Common &c) {
    c.o = gnn_ap_opts{};
    if (opts_in) c.o = *opts_in;
    if (N < 0 || d < 0 || N > INT32_MAX || d > INT32_MAX) return GNN_ERR_INVALID_ARG;
    if (binop < GNN_BIN_ADD || binop > GNN_BIN_COPY_RHS) return GNN_ERR_INVALID_ARG;
    if (c.o.edge_width != 0 && c.o.edge_width != 1 && c.o.edge_width != d) return GNN_ERR_INVALID_ARG;
    c.ewide = c.o.edge_width != 1 || d == 1;
    const int64_t ew = c.o.edge_width == 1 ? 1 : d;
    c.ldv = c.o.ldv ? c.o.ldv : d;
    c.lde = c.o.lde ? c.o.lde : ew;
    c.ldo = c.o.ldo ? c.o.ldo : d;
    if (c.ldv < d || c.lde < ew || c.ldo < d) return GNN_ERR_INVALID_ARG;
    if (c.o.plan && (c.o.plan->n_rows != N || c.o.plan->indptr_is_64 != (c.o.indptr_is_64 ? 1 : 0))) return GNN_ERR_INVALID_ARG;
    c.stream = static_cast<hipStream_t>(c.o.stream);
    return GNN_OK;
}

template <int BIN, int RED, int VEC>
void launch_fwd_ew(bool ewide, dim3 grid, hipStream_t stream, const ApArgs &a) {
    if (BIN == GNN_BIN_COPY_LHS || ewide) ap_fwd_kernel<BIN, RED, VEC, true><<<grid, kBlockThreads, 0, stream>>>(a);
    else ap_fwd_kernel<BIN, RED, VEC, false><<<grid, kBlockThreads, 0, stream>>>(a);
}
template <int BIN, int RED>
void launch_fwd_vec(int vec, bool ewide, dim3 grid, hipStream_t stream, const ApArgs &a) {
    if (vec == 4) launch_fwd_ew<BIN, RED, 4>(ewide, grid, stream, a);
    else launch_fwd_ew<BIN, RED, 1>(ewide, grid, stream, a);
}
template <int BIN>
void launch_fwd_red(int red, int vec, bool ewide, dim3 grid, hipStream_t stream, const ApArgs &a) {
    if (red == GNN_RED_SUM) launch_fwd_vec<BIN, GNN_RED_SUM>(vec, ewide, grid, stream, a);
    else if (red == GNN_RED_MAX) launch_fwd_vec<BIN, GNN_RED_MAX>(vec, ewide, grid, stream, a);
    else launch_fwd_vec<BIN, GNN_RED_MIN>(vec, ewide, grid, stream, a);
}
void launch_fwd(int bin, int red, int vec, bool ewide, dim3 grid, hipStream_t stream, const ApArgs &a) {
    switch (bin) {
        case GNN_BIN_ADD: launch_fwd_red<GNN_BIN_ADD>(red, vec, ewide, grid, stream, a); break;
        case GNN_BIN_SUB: launch_fwd_red<GNN_BIN_SUB>(red, vec, ewide, grid, stream, a); break;
        case GNN_BIN_MUL: launch_fwd_red<GNN_BIN_MUL>(red, vec, ewide, grid, stream, a); break;
        case GNN_BIN_DIV: launch_fwd_red<GNN_BIN_DIV>(red, vec, ewide, grid, stream, a); break;
        case GNN_BIN_COPY_LHS: launch_fwd_red<GNN_BIN_COPY_LHS>(red, vec, ewide, grid, stream, a); break;
        default: launch_fwd_red<GNN_BIN_COPY_RHS>(red, vec, ewide, grid, stream, a); break;
    }
}

__global__ void unpad_rows_kernel(const float *__restrict__ val, const int32_t *__restrict__ arg, int64_t ld_src,
                                  float *__restrict__ out, int64_t ldo, int32_t *__restrict__ arg_out, int64_t N, int d);

int run_ap_fwd(const void *indptr, const int32_t *indices, const float *fV, const float *fE, float *fO, int32_t *arg_e,
               int64_t N, int64_t d, int binop, int reduce, const gnn_ap_opts *opts_in) {
    Common c;
    int rc = check_common(opts_in, N, d, binop, c);
    if (rc != GNN_OK) return rc;
    if (reduce < GNN_RED_SUM || reduce > GNN_RED_MIN) return GNN_ERR_INVALID_ARG;
    if (reduce == GNN_RED_SUM && arg_e) return GNN_ERR_INVALID_ARG;
    if (N == 0 || d == 0) return GNN_OK;
    const bool use_v = binop != GNN_BIN_COPY_RHS, use_e = binop != GNN_BIN_COPY_LHS;
    if (!indptr || !fO || (use_v && !fV) || (use_e && !fE)) return GNN_ERR_INVALID_ARG;
    if (!aligned4(fO) || (use_v && !aligned4(fV)) || (use_e && !aligned4(fE)) || (arg_e && !aligned4(arg_e))) return GNN_ERR_INVALID_ARG;
    gnn_plan *plan = c.o.plan;
    if (plan && plan->n_edges > 0 && !indices) return GNN_ERR_INVALID_ARG;
    if (reduce != GNN_RED_SUM && plan && plan->n_edges > INT32_MAX) return GNN_ERR_UNSUPPORTED;
    (void)hipGetLastError();

    const bool wide = use_e && c.ewide;

    // The sum of the neighbours' vectors, plain or weighted by a scalar per edge in CSR order, is
    // the operation of the sum-only path (Alg. 1): that path has the layouts tuned for it.
    // A scalar operand that is strided or reached through an edge-id map (the backward pass over the
    // transposed graph) is first brought into CSR order, one pass over E values into a plan-owned
    // array: the sliced launches then stream it instead of repeating random 4-byte reads per slice.
    if (reduce == GNN_RED_SUM && (binop == GNN_BIN_COPY_LHS || (binop == GNN_BIN_MUL && !wide))) {
        const float *w = nullptr;
        if (binop == GNN_BIN_MUL) {
            w = fE;
            if (c.o.edge_ids || c.lde != 1) {
                w = nullptr;
                if (plan && plan->n_edges > 0) {
                    rc = gnn_plan_edge_operand(plan, fE, c.lde, c.o.edge_ids, c.stream, &w);
                    if (rc != GNN_OK) return rc;
                }
            }
        }
        if (binop == GNN_BIN_COPY_LHS || w) rc = GNN_OK; else rc = GNN_ERR_UNSUPPORTED;
        gnn_opts g{};
        g.dtype = GNN_F32;
        g.indptr_is_64 = c.o.indptr_is_64;
        g.ldx = c.ldv;
        g.ldy = c.ldo;
        g.stream = c.o.stream;
        g.plan = plan;
        g.flags = c.o.flags;
        g.max_slices = c.o.max_slices;
        if (rc == GNN_OK) rc = gnn_aggregate_fwd(indptr, indices, w, fV, fO, N, d, GNN_SUM, &g);
        if (rc != GNN_ERR_UNSUPPORTED) return rc;  // shapes that path does not take go through the kernel below
    }

    int vec = 4;
    if (d % 4 || c.ldo % 4 || !aligned16(fO)) vec = 1;
    if (use_v && (c.ldv % 4 || !aligned16(fV))) vec = 1;
    if (wide && (c.lde % 4 || !aligned16(fE))) vec = 1;
    if (arg_e && !aligned16(arg_e)) vec = 1;
    // Staged call: a width or strides that forbid 16-byte accesses on a gather-bound call of a large
    // graph.  f_V is copied into padded rows anyway (below); the results are computed in plan-owned
    // rows of roundup(d, 4) columns as well and copied to the caller's arrays at the end, so the
    // kernel runs its 16-byte instantiation (copylhs / max d = 33: 4.3 -> 3.7 ms, d = 101: 10.1 -> 7.9).
    const int64_t d4 = (d + 3) / 4 * 4;
    bool staged = false;
    if (vec == 1 && use_v && !wide && plan && plan->n_edges >= 16 * N && N * d * 4 >= (int64_t(1) << 20) && d * 4 > 128) {
        const gnn_layout Ls = gnn_choose_layout(plan, N, d, 4, c.ldv, reinterpret_cast<uintptr_t>(fV) % 128 == 0, c.o.flags,
                                                c.o.max_slices);
        staged = Ls.padded_copy;
    }
    if (staged) vec = 4;

    ApArgs a{};
    a.indptr = indptr;
    a.indices = indices;
    a.eid = c.o.edge_ids;
    a.fV = fV;
    a.fE = fE;
    a.out = fO;
    a.arg_out = arg_e;
    a.ld_arg = d;
    a.ldv = c.ldv;
    a.lde = c.lde;
    a.ldo = c.ldo;
    a.d = int32_t(d);
    a.ip64 = c.o.indptr_is_64 ? 1 : 0;
    const bool has_hub = plan && plan->n_chunks > 0;
    if (has_hub) {
        a.ldp = gnn_partial_ld(d);
        rc = gnn_plan_reserve(plan, 2 * a.ldp);  // values and winners
        if (rc != GNN_OK) return rc;
        a.pval = static_cast<float *>(plan->scratch);
        a.parg = reinterpret_cast<int32_t *>(a.pval + plan->n_chunks * a.ldp);
    }

    // Gather-bound calls (no full-width edge operand) get the layout of the sum-only hot path:
    // rows copied to an odd number of 128-byte lines when the plan says column slices pay, and
    // one-line column slices spread over the XCD L2s, 8 / 4 / 2 / 1 slices per launch.
    // Not with an edge-id map on a scalar edge operand (every slice would repeat the random 4-byte
    // reads: measured 10.5 -> 16.6 ms at d = 100), nor for max / min with a scalar operand (the
    // repeated weight stream and winner bookkeeping cost more than the hits bring: 8.4 -> 9.0 ms).
    bool sliced = false;
    const bool slice_ok = !use_e || (!wide && !c.o.edge_ids && reduce == GNN_RED_SUM) || c.o.max_slices > 1;
    if (use_v && !wide && vec == 4 && plan && plan->n_edges > 0 && (slice_ok || staged)) {
        gnn_layout L = gnn_choose_layout(plan, N, d, 4, c.ldv, reinterpret_cast<uintptr_t>(fV) % 128 == 0, c.o.flags,
                                         c.o.max_slices);
        if (!slice_ok) L.slices_wanted = false;  // staged only: the copy, not the slices
        if (L.padded_copy && d * 4 > 128) {  // rows of one line gain nothing from a copy in their own order
            const int64_t copy_bytes = (N * L.ld_pad * 4 + 255) / 256 * 256;
            const int64_t tmp_bytes = (N * d4 * 4 + 255) / 256 * 256;
            rc = gnn_plan_padded(plan, copy_bytes + (staged ? tmp_bytes * (arg_e ? 2 : 1) : 0));
            if (rc != GNN_OK) return rc;
            rc = gnn_pad_rows_f32(fV, c.ldv, static_cast<float *>(plan->padded), L.ld_pad, N, d, c.stream);
            if (rc != GNN_OK) return rc;
            a.fV = static_cast<const float *>(plan->padded);
            a.ldv = L.ld_pad;
            if (staged) {
                char *base = static_cast<char *>(plan->padded) + copy_bytes;
                a.out = reinterpret_cast<float *>(base);
                a.ldo = d4;
                if (arg_e) {
                    a.arg_out = reinterpret_cast<int32_t *>(base + tmp_bytes);
                    a.ld_arg = d4;
                }
            }
        }
        const int64_t line = 32;  // floats per 128-byte line
        const bool lines_ok = a.ldv % line == 0 && reinterpret_cast<uintptr_t>(a.fV) % 128 == 0;
        const int64_t lines = (d + line - 1) / line;
        int64_t g16 = 1;
        while (g16 < 16 && (a.ldv / line) % (g16 * 2) == 0) g16 *= 2;
        const int64_t unit_lines = g16 >= 8 ? g16 / 4 : 1;  // even strides: wider slices (see aggregate.hip)
        const int64_t units = (lines + unit_lines - 1) / unit_lines;
        if (L.slices_wanted && lines_ok && units >= 2 && units <= 256 && c.o.max_slices != 1) {
            sliced = true;
            if (!(c.o.flags & GNN_FLAG_NO_COLD_HINTS)) {
                const int32_t *flagged = nullptr;
                rc = gnn_plan_cold_indices(plan, indices, (c.o.flags & GNN_FLAG_FORCE_COLD_HINTS) != 0, c.stream, &flagged);
                if (rc != GNN_OK) return rc;
                if (flagged) a.indices = flagged;
            }
            a.slab_cols = int32_t(unit_lines * line);
            const int log2_c = gnn_ilog2_ceil(a.slab_cols / vec);
            int64_t u0 = 0;
            while (u0 < units) {
                const int64_t s_max = c.o.max_slices > 0 ? c.o.max_slices : 8;
                int ls = 3;
                while (ls > 0 && ((int64_t(1) << ls) > units - u0 || (int64_t(1) << ls) > s_max)) --ls;
                a.col0 = int32_t(u0 * a.slab_cols);
                const int64_t end = int64_t(a.col0) + (int64_t(a.slab_cols) << ls);
                a.col_end = int32_t(end < d ? end : d);
                a.log2_slices = ls;
                const int64_t blocks = make_bins(a, plan, N, log2_c) << ls;
                if (blocks > INT32_MAX) return GNN_ERR_UNSUPPORTED;
                if (blocks > 0) {
                    launch_fwd(binop, reduce, vec, c.ewide, dim3(static_cast<unsigned>(blocks)), c.stream, a);
                    if (hipGetLastError() != hipSuccess) return GNN_ERR_LAUNCH;
                }
                u0 += int64_t(1) << ls;
            }
        }
    }
    if (!sliced) {
        const int64_t strips = (d + vec - 1) / vec;
        const int log2_c = strips >= 64 ? 6 : gnn_ilog2_ceil(strips);
        const int64_t slab_cols = (int64_t(1) << log2_c) * vec;
        const int64_t n_slabs = (d + slab_cols - 1) / slab_cols;
        if (n_slabs > 65535) return GNN_ERR_UNSUPPORTED;
        a.slab_cols = int32_t(slab_cols);
        a.col0 = 0;
        a.col_end = int32_t(d);
        a.log2_slices = 0;
        const int64_t blocks = make_bins(a, plan, N, log2_c);
        if (blocks > INT32_MAX) return GNN_ERR_UNSUPPORTED;
        if (blocks > 0) {
            dim3 grid(static_cast<unsigned>(blocks), static_cast<unsigned>(n_slabs));
            launch_fwd(binop, reduce, vec, c.ewide, grid, c.stream, a);
            if (hipGetLastError() != hipSuccess) return GNN_ERR_LAUNCH;
        }
    }
    if (has_hub) {
        const int64_t hub_begin = plan->bin_offsets[plan->n_bins - 1];
        dim3 grid(static_cast<unsigned>(plan->n_hub_rows));
        const int32_t *hub_rows = plan->row_perm + hub_begin;
        if (reduce == GNN_RED_SUM)
            ap_hub_finalize_kernel<GNN_RED_SUM><<<grid, 256, 0, c.stream>>>(hub_rows, plan->n_hub_rows, plan->hub_chunk_offsets, a.pval, a.parg, a.ldp, a.out, a.ldo, a.arg_out, a.ld_arg, int(d));
        else if (reduce == GNN_RED_MAX)
            ap_hub_finalize_kernel<GNN_RED_MAX><<<grid, 256, 0, c.stream>>>(hub_rows, plan->n_hub_rows, plan->hub_chunk_offsets, a.pval, a.parg, a.ldp, a.out, a.ldo, a.arg_out, a.ld_arg, int(d));
        else
            ap_hub_finalize_kernel<GNN_RED_MIN><<<grid, 256, 0, c.stream>>>(hub_rows, plan->n_hub_rows, plan->hub_chunk_offsets, a.pval, a.parg, a.ldp, a.out, a.ldo, a.arg_out, a.ld_arg, int(d));
        if (hipGetLastError() != hipSuccess) return GNN_ERR_LAUNCH;
    }
    if (a.out != fO) {  // staged call: hand the results over
        int64_t blocks = (N * d + 255) / 256;
        if (blocks > (int64_t(1) << 17)) blocks = int64_t(1) << 17;
        unpad_rows_kernel<<<static_cast<unsigned>(blocks), 256, 0, c.stream>>>(a.out, a.arg_out, a.ldo, fO, c.ldo, arg_e, N, int(d));
        if (hipGetLastError() != hipSuccess) return GNN_ERR_LAUNCH;
    }
    return GNN_OK;
}

template <int BIN, int VEC, bool EWIDE>
void launch_edge_masked(bool masked, dim3 grid, hipStream_t stream, const ApArgs &a) {
    if (masked) ap_bwd_edge_kernel<BIN, VEC, EWIDE, true><<<grid, kBlockThreads, 0, stream>>>(a);
    else ap_bwd_edge_kernel<BIN, VEC, EWIDE, false><<<grid, kBlockThreads, 0, stream>>>(a);
}
template <int BIN>
void launch_edge_bin(int vec, bool ewide, bool masked, dim3 grid, hipStream_t stream, const ApArgs &a) {
    if (vec == 4) {
        if (ewide) launch_edge_masked<BIN, 4, true>(masked, grid, stream, a);
        else launch_edge_masked<BIN, 4, false>(masked, grid, stream, a);
    } else {
        if (ewide) launch_edge_masked<BIN, 1, true>(masked, grid, stream, a);
        else launch_edge_masked<BIN, 1, false>(masked, grid, stream, a);
    }
}

// Results of a staged call go from the padded rows they were computed in to the caller's arrays.
__global__ void __launch_bounds__(256) unpad_rows_kernel(const float *__restrict__ val, const int32_t *__restrict__ arg,
                                                         int64_t ld_src, float *__restrict__ out, int64_t ldo,
                                                         int32_t *__restrict__ arg_out, int64_t N, int d) {
    const int64_t total = N * d;
    const int64_t stride = int64_t(gridDim.x) * blockDim.x;
    for (int64_t t = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; t < total; t += stride) {
        const int64_t r = t / d;
        const int c = int(t - r * d);
        out[r * ldo + c] = val[r * ld_src + c];
        if (arg_out) arg_out[r * int64_t(d) + c] = arg[r * ld_src + c];
    }
}

// dst[r, 0..ld_dst) = src[r, 0..d) followed by zeros (ld_dst a multiple of 4 floats, dst 16-byte aligned).
__global__ void __launch_bounds__(256) pad_zero_rows_kernel(const float *__restrict__ src, int64_t ld_src,
                                                            float *__restrict__ dst, int64_t ld_dst, int64_t N, int d) {
    const int quads = int(ld_dst / 4);
    int log2_tpr = 0;
    while ((1 << log2_tpr) < quads && log2_tpr < 8) ++log2_tpr;
    const int tpr = 1 << log2_tpr;
    const int64_t rows_per_block = blockDim.x >> log2_tpr;
    for (int64_t row = int64_t(blockIdx.x) * rows_per_block + (threadIdx.x >> log2_tpr); row < N;
         row += int64_t(gridDim.x) * rows_per_block) {
        const float *in = src + row * ld_src;
        for (int q = threadIdx.x & (tpr - 1); q < quads; q += tpr) {
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = 4 * q + i < d ? in[4 * q + i] : 0.0f;
            *reinterpret_cast<float4 *>(dst + row * ld_dst + 4 * q) = make_float4(v[0], v[1], v[2], v[3]);
        }
    }
}

}  // namespace

extern "C" GNN_API int gnn_ap_fwd(const void *indptr, const int32_t *indices, const float *fV, const float *fE, float *fO,
                                  int32_t *arg_e, int64_t N, int64_t d, int binop, int reduce, const gnn_ap_opts *opts) {
    return run_ap_fwd(indptr, indices, fV, fE, fO, arg_e, N, d, binop, reduce, opts);
}

extern "C" GNN_API int gnn_ap_bwd_vertex(const void *indptr_t, const int32_t *indices_t, const float *dO, const float *fE,
                                         float *dfV, int64_t N, int64_t d, int binop, const gnn_ap_opts *opts) {
    Common c;
    int rc = check_common(opts, N, d, binop, c);
    if (rc != GNN_OK) return rc;
    if (N == 0 || d == 0) return GNN_OK;
    if (!dfV || !aligned4(dfV)) return GNN_ERR_INVALID_ARG;
    // the gathered operand is dO (stride ldo), the output dfV (stride ldv): swap the two strides
    gnn_ap_opts t = c.o;
    t.ldv = c.ldo;
    t.ldo = c.ldv;
    switch (binop) {
        case GNN_BIN_COPY_RHS:
            (void)hipGetLastError();
            fill_rows_kernel<<<grid_1d(N * d), 256, 0, c.stream>>>(dfV, c.ldv, N, int(d), 0.0f);
            return hipGetLastError() == hipSuccess ? GNN_OK : GNN_ERR_LAUNCH;
        case GNN_BIN_MUL:
        case GNN_BIN_DIV:
            return run_ap_fwd(indptr_t, indices_t, dO, fE, dfV, nullptr, N, d, binop, GNN_RED_SUM, &t);
        default:  // add, sub, copylhs: d/dx = 1
            return run_ap_fwd(indptr_t, indices_t, dO, nullptr, dfV, nullptr, N, d, GNN_BIN_COPY_LHS, GNN_RED_SUM, &t);
    }
}

extern "C" GNN_API int gnn_ap_bwd_vertex_arg(const int32_t *indices, const int32_t *arg_e, const float *dO, const float *fE,
                                             float *dfV, int64_t n_vertex_rows, int64_t N, int64_t d, int binop,
                                             const gnn_ap_opts *opts) {
    Common c;
    gnn_ap_opts o{};
    if (opts) o = *opts;
    o.plan = nullptr;  // not used here
    int rc = check_common(&o, N, d, binop, c);
    if (rc != GNN_OK) return rc;
    if (n_vertex_rows < 0) return GNN_ERR_INVALID_ARG;
    if (d == 0) return GNN_OK;
    if (!dfV || !aligned4(dfV)) return GNN_ERR_INVALID_ARG;
    (void)hipGetLastError();
    if (n_vertex_rows > 0) fill_rows_kernel<<<grid_1d(n_vertex_rows * d), 256, 0, c.stream>>>(dfV, c.ldv, n_vertex_rows, int(d), 0.0f);
    if (hipGetLastError() != hipSuccess) return GNN_ERR_LAUNCH;
    if (N == 0 || binop == GNN_BIN_COPY_RHS) return GNN_OK;
    const bool need_y = binop == GNN_BIN_MUL || binop == GNN_BIN_DIV;
    if (!indices || !arg_e || !dO || (need_y && !fE)) return GNN_ERR_INVALID_ARG;
    const unsigned grid = grid_1d(N * d);
    const int ew = c.ewide ? 1 : 0;
    if (binop == GNN_BIN_MUL)
        ap_scatter_arg_kernel<GNN_BIN_MUL><<<grid, 256, 0, c.stream>>>(indices, c.o.edge_ids, arg_e, dO, c.ldo, fE, c.lde, ew, dfV, c.ldv, N, int(d));
    else if (binop == GNN_BIN_DIV)
        ap_scatter_arg_kernel<GNN_BIN_DIV><<<grid, 256, 0, c.stream>>>(indices, c.o.edge_ids, arg_e, dO, c.ldo, fE, c.lde, ew, dfV, c.ldv, N, int(d));
    else
        ap_scatter_arg_kernel<GNN_BIN_COPY_LHS><<<grid, 256, 0, c.stream>>>(indices, c.o.edge_ids, arg_e, dO, c.ldo, fE, c.lde, ew, dfV, c.ldv, N, int(d));
    return hipGetLastError() == hipSuccess ? GNN_OK : GNN_ERR_LAUNCH;
}

extern "C" GNN_API int gnn_ap_bwd_edge(const void *indptr, const int32_t *indices, const int32_t *arg_e, const float *fV,
                                       const float *fE, const float *dO, float *dfE, int64_t N, int64_t d, int binop,
                                       const gnn_ap_opts *opts) {
    Common c;
    int rc = check_common(opts, N, d, binop, c);
    if (rc != GNN_OK) return rc;
    if (binop == GNN_BIN_COPY_LHS) return GNN_ERR_INVALID_ARG;
    if (N == 0 || d == 0) return GNN_OK;
    const bool need_x = binop == GNN_BIN_MUL || binop == GNN_BIN_DIV, need_y = binop == GNN_BIN_DIV;
    if (!indptr || !dO || !dfE || (need_x && !fV) || (need_y && !fE)) return GNN_ERR_INVALID_ARG;
    if (!aligned4(dO) || !aligned4(dfE) || (need_x && !aligned4(fV)) || (need_y && !aligned4(fE)) || (arg_e && !aligned4(arg_e)))
        return GNN_ERR_INVALID_ARG;
    gnn_plan *plan = c.o.plan;
    if (plan && plan->n_edges > 0 && !indices) return GNN_ERR_INVALID_ARG;
    if (arg_e && plan && plan->n_edges > INT32_MAX) return GNN_ERR_UNSUPPORTED;
    (void)hipGetLastError();

    int vec = 4;
    if (d % 4 || c.ldo % 4 || !aligned16(dO)) vec = 1;
    if (need_x && (c.ldv % 4 || !aligned16(fV))) vec = 1;
    if (c.ewide && (c.lde % 4 || !aligned16(dfE) || (need_y && !aligned16(fE)))) vec = 1;
    if (arg_e && !aligned16(arg_e)) vec = 1;

    // A scalar edge gradient is a dot product over the columns, so rows whose width or stride
    // forbids 16-byte loads are first copied into plan-owned rows of a multiple of four floats, padded
    // with zeros (they add +0 to every sum): d = 33 on 2.45 M vertices 14.2 -> 4.3 ms.
    int64_t d_run = d, ldv_run = c.ldv, ldo_run = c.ldo;
    if (vec == 1 && !c.ewide && !arg_e && plan && plan->n_edges >= 16 * N && N * d * 4 >= (int64_t(1) << 20)) {
        const int64_t d4 = (d + 3) / 4 * 4;
        rc = gnn_plan_padded(plan, (need_x ? 2 : 1) * N * d4 * 4);
        if (rc != GNN_OK) return rc;
        float *dO_pad = static_cast<float *>(plan->padded);
        float *fV_pad = dO_pad + N * d4;
        const int quads = int(d4 / 4);
        int log2_tpr = 0;
        while ((1 << log2_tpr) < quads && log2_tpr < 8) ++log2_tpr;
        int64_t blocks = (N + (256 >> log2_tpr) - 1) / (256 >> log2_tpr);
        if (blocks > (int64_t(1) << 17)) blocks = int64_t(1) << 17;
        pad_zero_rows_kernel<<<static_cast<unsigned>(blocks), 256, 0, c.stream>>>(dO, c.ldo, dO_pad, d4, N, int(d));
        if (need_x) pad_zero_rows_kernel<<<static_cast<unsigned>(blocks), 256, 0, c.stream>>>(fV, c.ldv, fV_pad, d4, N, int(d));
        if (hipGetLastError() != hipSuccess) return GNN_ERR_LAUNCH;
        dO = dO_pad;
        if (need_x) fV = fV_pad;
        d_run = d4; ldo_run = d4; if (need_x) ldv_run = d4;
        vec = 4;
    }

    const int64_t strips = (d_run + vec - 1) / vec;
    const int log2_c = strips >= 64 ? 6 : gnn_ilog2_ceil(strips);

    ApArgs a{};
    a.indptr = indptr;
    a.indices = indices;
    a.eid = c.o.edge_ids;
    a.fV = fV;
    a.fE = fE;
    a.dO = dO;
    a.out = dfE;
    a.arg_in = arg_e;
    a.ldv = ldv_run;
    a.lde = c.lde;
    a.ldo = ldo_run;
    a.d = int32_t(d_run);
    a.ip64 = c.o.indptr_is_64 ? 1 : 0;
    const int64_t blocks = make_bins(a, plan, N, log2_c);
    if (blocks > INT32_MAX) return GNN_ERR_UNSUPPORTED;
    if (blocks == 0) return GNN_OK;
    dim3 grid(static_cast<unsigned>(blocks));
    const bool masked = arg_e != nullptr;
    switch (binop) {
        case GNN_BIN_ADD: launch_edge_bin<GNN_BIN_ADD>(vec, c.ewide, masked, grid, c.stream, a); break;
        case GNN_BIN_SUB: launch_edge_bin<GNN_BIN_SUB>(vec, c.ewide, masked, grid, c.stream, a); break;
        case GNN_BIN_MUL: launch_edge_bin<GNN_BIN_MUL>(vec, c.ewide, masked, grid, c.stream, a); break;
        case GNN_BIN_DIV: launch_edge_bin<GNN_BIN_DIV>(vec, c.ewide, masked, grid, c.stream, a); break;
        default: launch_edge_bin<GNN_BIN_COPY_RHS>(vec, c.ewide, masked, grid, c.stream, a); break;
    }
    return hipGetLastError() == hipSuccess ? GNN_OK : GNN_ERR_LAUNCH;
}
