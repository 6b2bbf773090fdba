// Neighbour aggregation kernels (Section 4.1, Algorithm 1) for gfx950.
//
//   Y[v, :] = dst_scale(v) * sum_{e in row v} coef(e) * X[indices[e], :]
//
// The same kernel serves the forward pass (CSR by destination) and the
// backward pass (the transposed graph): only the arrays and the scale modes
// differ.  This is HBM/cache-bandwidth-bound gather work, not a dense
// contraction, so there is no MFMA here; the design points are
//   * a 64-lane wavefront is cut into row groups of G lanes; a group owns one
//     output row (one owner per row, as in the paper, so no atomics).  Inside a
//     group, C lanes span the feature row with 16/8/4-byte loads and SR = G/C
//     "edge slots" walk the neighbour list SR edges at a time; the slots are
//     combined with wavefront shuffles at the end of the row.  G, SR come from
//     the degree bin of the row (light rows: many rows per wavefront; heavy
//     rows: the whole wavefront on one row).
//   * neighbour ids (and per-edge coefficients) are fetched as one coalesced
//     tile per group and handed to the slots by cross-lane shuffles, so the
//     index stream is read once, fully coalesced;
//   * accumulation stays in registers for the whole neighbour loop and the
//     output row is written once (the loop order of Algorithm 3);
//   * rows of the hub bin are cut into pieces reduced by different wavefronts
//     into an fp32 scratch; a second kernel adds the pieces in fixed order;
//   * workgroup b of a launch gathers only the 128-byte column slice b % S of
//     the rows, so that the private L2 of the XCD it runs on holds one line of
//     many rows instead of whole rows of few; for a large graph the gathered
//     matrix is first copied into a plan-owned layout made for that: one table
//     per slice, rows by descending gather count, a dense table for a short last
//     line (run_aggregate below).
#include <mutex>

#include "common.h"

// Hub partial sums of gnn_aggregate_fwd_noalloc, the entry point that allocates nothing: one array
// per GPU, part of the loaded code object, held until the process ends.  In host code this name
// only stands for the symbol; the device address is looked up once per device and kept
// (static_scratch_of_current_device), and only that address is ever handed to a kernel.
static __device__ __align__(256) float scratch[GNN_NOALLOC_SCRATCH_BYTES / sizeof(float)];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
float *g_scratch_ptr[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device (looked up on the first call there).
int static_scratch_of_current_device(float **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GNN_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return GNN_ERR_LAUNCH;
        g_scratch_ptr[dev] = static_cast<float *>(p);
    }
    *out = g_scratch_ptr[dev];
    return GNN_OK;
}

constexpr int kBlockThreads = 256;
constexpr int kWavesPerBlock = kBlockThreads / 64;

enum ScaleMode : int { kScaleNone = 0, kScaleInv = 1, kScaleRsqrt = 2, kScaleInvPlus1 = 3 };
enum SelfMode : int { kSelfNone = 0, kSelfPlain = 1, kSelfInvPlus1 = 2 };  // own row added to the sum
constexpr int kKindHubPieces = GNN_BIN_HUB_PIECES;
using BinDesc = gnn_bin_desc;

struct AggArgs {
    const void *indptr;
    const int32_t *indices;
    const float *w;
    const void *X;
    void *Y;
    int64_t ldx, ldy;
    int32_t F;
    int32_t ip64;
    const int32_t *row_perm;    // nullptr: identity
    const float *edge_scale;    // per-edge factor 1/deg or 1/sqrt(deg) of the gathered vertex, or nullptr
    int32_t dst_mode;
    int32_t self_mode;          // SelfMode: add the row's own gathered vector (GraphSAGE-GCN aggregator)
    const int32_t *col_counts;  // per-vertex column counts of the plan (self term of the backward pass)
    const int64_t *chunks;      // hub pieces (row, e_begin, e_end)
    float *partial;             // [n_chunks, ldp] fp32
    int64_t ldp;
    int32_t n_bins;
    int32_t log2_slices;  // column slices; workgroup b serves slice b % n_slices (see run_aggregate)
    int32_t slice_cols;   // columns per slice (the last slice of a launch may hold fewer)
    int32_t store_vec;    // widest store the output rows allow (elements, <= VEC)
    const int32_t *row_map;  // row of the gathered table that holds vertex v (rank layout), or nullptr: v
    const int64_t *p_indptr;  // rank layout: edge range of the row at position i of row_perm within `indices`
    const int64_t *p_chunks;  // rank layout: hub pieces (row, begin, end, original - plan-order position)
    int32_t cold_on;      // honour the cold flag (bit 31) of the indices
    int32_t warm_rank;    // rank layout: sources of rank >= this are cold too (INT32_MAX: none)
    int64_t slice_stride;  // > 0: slice-major copy, slice s of the launch reads the table at X + s * slice_stride elements
    const void *X_tail;   // dense tail table (see gnn_layout), read by slice `tail_slice` of the launch
    int64_t ld_tail;
    int32_t tail_slice;   // -1: none
    const float *bias;    // fused layer epilogue: per-column bias added to the scaled row, or nullptr
    int32_t relu;         // fused layer epilogue: rectifier after the bias
    BinDesc bins[GNN_MAX_BINS + 1];
};

// ------------------------------------------------------------ element access
struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(uint32_t(b) << 16); }

// Round to nearest even; NaN stays NaN (quiet).
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return uint16_t((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return uint16_t(u >> 16);
}

template <typename T, int VEC> struct VecIO;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

template <> struct VecIO<float, 4> {
    static __device__ __forceinline__ void load(const float *p, float (&v)[4]) {
        float4 t = *reinterpret_cast<const float4 *>(p); v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
    static __device__ __forceinline__ void load_nt(const float *p, float (&v)[4]) {
        f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p)); v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
    // Output rows are written once and not read again by this kernel: non-temporal stores keep
    // them from displacing gathered rows in the L2 (measured: +0.5..1 %).
    static __device__ __forceinline__ void store(float *p, const float (&v)[4]) {
        f32x4 t = {v[0], v[1], v[2], v[3]};
        __builtin_nontemporal_store(t, reinterpret_cast<f32x4 *>(p));
    }
};
template <> struct VecIO<float, 2> {
    static __device__ __forceinline__ void load(const float *p, float (&v)[2]) {
        float2 t = *reinterpret_cast<const float2 *>(p); v[0] = t.x; v[1] = t.y;
    }
    static __device__ __forceinline__ void load_nt(const float *p, float (&v)[2]) {
        f32x2 t = __builtin_nontemporal_load(reinterpret_cast<const f32x2 *>(p)); v[0] = t.x; v[1] = t.y;
    }
    static __device__ __forceinline__ void store(float *p, const float (&v)[2]) {
        f32x2 t = {v[0], v[1]};
        __builtin_nontemporal_store(t, reinterpret_cast<f32x2 *>(p));
    }
};
template <> struct VecIO<float, 1> {
    static __device__ __forceinline__ void load(const float *p, float (&v)[1]) { v[0] = *p; }
    static __device__ __forceinline__ void load_nt(const float *p, float (&v)[1]) { v[0] = __builtin_nontemporal_load(p); }
    static __device__ __forceinline__ void store(float *p, const float (&v)[1]) { __builtin_nontemporal_store(v[0], p); }
};
template <> struct VecIO<bf16_t, 8> {
    static __device__ __forceinline__ void unpack(const uint32_t (&w)[4], float (&v)[8]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) { v[2 * i] = __uint_as_float(w[i] << 16); v[2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u); }
    }
    static __device__ __forceinline__ void load(const bf16_t *p, float (&v)[8]) {
        uint4 t = *reinterpret_cast<const uint4 *>(p);
        uint32_t w[4] = {t.x, t.y, t.z, t.w};
        unpack(w, v);
    }
    static __device__ __forceinline__ void load_nt(const bf16_t *p, float (&v)[8]) {
        u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
        uint32_t w[4] = {t.x, t.y, t.z, t.w};
        unpack(w, v);
    }
    static __device__ __forceinline__ void store(bf16_t *p, const float (&v)[8]) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = uint32_t(f32_to_bf16(v[2 * i])) | (uint32_t(f32_to_bf16(v[2 * i + 1])) << 16);
        u32x4 t = {w[0], w[1], w[2], w[3]};
        __builtin_nontemporal_store(t, reinterpret_cast<u32x4 *>(p));
    }
};
template <> struct VecIO<bf16_t, 4> {
    static __device__ __forceinline__ void load(const bf16_t *p, float (&v)[4]) {
        uint2 t = *reinterpret_cast<const uint2 *>(p);
        v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xFFFF0000u);
        v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xFFFF0000u);
    }
    static __device__ __forceinline__ void load_nt(const bf16_t *p, float (&v)[4]) {
        u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(p));
        v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xFFFF0000u);
        v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xFFFF0000u);
    }
    static __device__ __forceinline__ void store(bf16_t *p, const float (&v)[4]) {
        u32x2 t;
        t.x = uint32_t(f32_to_bf16(v[0])) | (uint32_t(f32_to_bf16(v[1])) << 16);
        t.y = uint32_t(f32_to_bf16(v[2])) | (uint32_t(f32_to_bf16(v[3])) << 16);
        __builtin_nontemporal_store(t, reinterpret_cast<u32x2 *>(p));
    }
};
template <> struct VecIO<bf16_t, 2> {
    static __device__ __forceinline__ void load(const bf16_t *p, float (&v)[2]) {
        uint32_t t = *reinterpret_cast<const uint32_t *>(p);
        v[0] = __uint_as_float(t << 16); v[1] = __uint_as_float(t & 0xFFFF0000u);
    }
    static __device__ __forceinline__ void load_nt(const bf16_t *p, float (&v)[2]) {
        uint32_t t = __builtin_nontemporal_load(reinterpret_cast<const uint32_t *>(p));
        v[0] = __uint_as_float(t << 16); v[1] = __uint_as_float(t & 0xFFFF0000u);
    }
    static __device__ __forceinline__ void store(bf16_t *p, const float (&v)[2]) {
        __builtin_nontemporal_store(uint32_t(f32_to_bf16(v[0])) | (uint32_t(f32_to_bf16(v[1])) << 16), reinterpret_cast<uint32_t *>(p));
    }
};
template <> struct VecIO<bf16_t, 1> {
    static __device__ __forceinline__ void load(const bf16_t *p, float (&v)[1]) { v[0] = bf16_to_f32(p->bits); }
    static __device__ __forceinline__ void load_nt(const bf16_t *p, float (&v)[1]) {
        v[0] = bf16_to_f32(__builtin_nontemporal_load(&p->bits));
    }
    static __device__ __forceinline__ void store(bf16_t *p, const float (&v)[1]) { __builtin_nontemporal_store(f32_to_bf16(v[0]), &p->bits); }
};

// A gathered strip stays in the registers the load filled (the packed bits: 16 bytes are four
// registers whether they hold 4 floats or 8 bf16) until it is added; unpacking at the load would
// keep U * VEC floats alive per lane and halve the occupancy of the bf16 kernels.
template <int BYTES> struct RawBits;
template <> struct RawBits<16> { typedef u32x4 type; };
template <> struct RawBits<8> { typedef u32x2 type; };
template <> struct RawBits<4> { typedef uint32_t type; };
template <> struct RawBits<2> { typedef uint16_t type; };

template <typename T, int VEC>
struct Strip {
    static constexpr int BYTES = int(sizeof(T)) * VEC;
    static constexpr int WORDS = BYTES >= 4 ? BYTES / 4 : 1;
    using raw_t = typename RawBits<BYTES>::type;
    static __device__ __forceinline__ raw_t load(const T *p) { return *reinterpret_cast<const raw_t *>(p); }
    static __device__ __forceinline__ raw_t load_nt(const T *p) {
        return __builtin_nontemporal_load(reinterpret_cast<const raw_t *>(p));
    }
    static __device__ __forceinline__ raw_t zero() {
        if constexpr (BYTES >= 8) { raw_t z; for (int i = 0; i < WORDS; ++i) z[i] = 0u; return z; }
        else return raw_t(0);
    }
    static __device__ __forceinline__ uint32_t word(const raw_t &r, int i) {
        if constexpr (BYTES >= 8) return r[i];
        else return uint32_t(r);
    }
    static __device__ __forceinline__ void unpack(const raw_t &r, float (&v)[VEC]) {
        if constexpr (sizeof(T) == 4) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) v[i] = __uint_as_float(word(r, i));
        } else if constexpr (VEC == 1) {
            v[0] = __uint_as_float(word(r, 0) << 16);
        } else {
#pragma unroll
            for (int i = 0; i < VEC / 2; ++i) {
                const uint32_t w = word(r, i);
                v[2 * i] = __uint_as_float(w << 16);
                v[2 * i + 1] = __uint_as_float(w & 0xFFFF0000u);
            }
        }
    }
};

// fp32 store of VEC consecutive values (hub partial sums are fp32 whatever T is)
template <int VEC>
__device__ __forceinline__ void store_f32(float *p, const float (&v)[VEC]) {
    if constexpr (VEC % 4 == 0) {
#pragma unroll
        for (int i = 0; i < VEC; i += 4) *reinterpret_cast<float4 *>(p + i) = make_float4(v[i], v[i + 1], v[i + 2], v[i + 3]);
    } else if constexpr (VEC == 2) {
        *reinterpret_cast<float2 *>(p) = make_float2(v[0], v[1]);
    } else {
        *p = v[0];
    }
}

// Output strip: one vector store when the output rows allow it, else narrower pieces; a
// partial last strip (padded gather source) writes only its valid columns.
template <typename T, int VEC>
__device__ __forceinline__ void store_strip(T *y, const float (&o)[VEC], int ncols, int store_vec) {
    if (ncols == VEC && store_vec == VEC) {
        VecIO<T, VEC>::store(y, o);
        return;
    }
    if constexpr (VEC >= 2) {
        if (ncols == VEC && store_vec * 2 == VEC) {
            float lo[VEC / 2], hi[VEC / 2];
#pragma unroll
            for (int i = 0; i < VEC / 2; ++i) { lo[i] = o[i]; hi[i] = o[VEC / 2 + i]; }
            VecIO<T, VEC / 2>::store(y, lo);
            VecIO<T, VEC / 2>::store(y + VEC / 2, hi);
            return;
        }
    }
    // single elements: plain stores, so that the L2 merges the pieces of a line before it is
    // written back (non-temporal 4-byte stores reach memory as partial lines)
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        if (i < ncols) {
            if constexpr (sizeof(T) == 4) *reinterpret_cast<float *>(y + i) = o[i];
            else reinterpret_cast<uint16_t *>(y + i)[0] = f32_to_bf16(o[i]);
        }
    }
}

__device__ __forceinline__ int64_t load_ip(const void *indptr, int ip64, int64_t i) {
    return ip64 ? static_cast<const int64_t *>(indptr)[i]
                : static_cast<int64_t>(static_cast<const int32_t *>(indptr)[i]);
}

__device__ __forceinline__ float scale_of(int mode, int64_t deg) { return gnn_row_factor(mode, deg); }

// The own-row term of a finalisation kernel reads the caller's matrix G, or -- when a producer wrote the
// gathered matrix straight into the plan's layout and no row-major copy exists -- that layout.
struct OwnRowSrc {
    const void *G;        // row-major [N, ldg], already offset to the first column of the launch; nullptr: use the layout
    int64_t ldg;
    const void *tbl;      // slice tables
    int64_t table_stride;
    int32_t main_cols;
    const void *tail;
    int64_t tail_ld;
    const int32_t *rank;
    int32_t col_off;      // first column of the launch within the matrix
};
template <typename T>
__device__ __forceinline__ float own_row_value(const OwnRowSrc &o, int64_t row, int colx) {
    constexpr int LINE = 128 / int(sizeof(T));
    float xs[1];
    if (o.G) {
        VecIO<T, 1>::load(static_cast<const T *>(o.G) + row * o.ldg + colx, xs);
    } else {
        const int col = o.col_off + colx;
        const int64_t r = o.rank[row];
        const T *q = col < o.main_cols ? static_cast<const T *>(o.tbl) + (col / LINE) * o.table_stride + r * LINE + col % LINE
                                       : static_cast<const T *>(o.tail) + r * o.tail_ld + (col - o.main_cols);
        VecIO<T, 1>::load(q, xs);
    }
    return xs[0];
}

// ---------------------------------------------------------------- main kernel
// T: storage type of X and Y.  VEC: elements per lane per load.  NPASS: feature
// passes (a lane owns NPASS strips of VEC columns, C*VEC apart).  COEF: edges
// carry a coefficient (explicit weight and/or a scale of the gathered vertex).
template <typename T, int VEC, int NPASS, bool COEF>
__global__ void __launch_bounds__(kBlockThreads) aggregate_kernel(const AggArgs a) {
    constexpr int U = NPASS >= 4 ? 2 : (NPASS >= 2 ? 4 : 8);  // edges in flight per slot
    const int lane = threadIdx.x & 63;
    const int wave_in_block = threadIdx.x >> 6;

    // which bin does this workgroup serve (wave-uniform scan of a tiny table)
    const int slice = int(blockIdx.x) & ((1 << a.log2_slices) - 1);
    const int64_t vblock = int64_t(blockIdx.x) >> a.log2_slices;
    const int col_base = slice * a.slice_cols;
    const int Fk = a.F - col_base < a.slice_cols ? a.F - col_base : a.slice_cols;  // columns of this slice
    if (Fk <= 0) return;
    int b = 0;
    for (int i = 1; i < a.n_bins; ++i)
        if (vblock >= a.bins[i].first_block) b = i;
    const BinDesc bin = a.bins[b];
    const int64_t wave_in_bin = (vblock - bin.first_block) * kWavesPerBlock + wave_in_block;

    const int G = 1 << bin.log2_g;
    const int SR = 1 << bin.log2_sr;
    const int log2_c = bin.log2_g - bin.log2_sr;
    const int C = 1 << log2_c;
    const int lane_in_g = lane & (G - 1);
    const int gbase = lane - lane_in_g;
    const int s = lane_in_g >> log2_c;  // edge slot of this lane
    const int c = lane_in_g & (C - 1);  // feature strip of this lane

    // the row (or hub piece) this group owns
    // e0..e1 index `indices`; the per-edge streams of the caller (weights, factors) live at e + wdelta
    int64_t e0 = 0, e1 = 0, row = -1, row_len = 0, wdelta = 0;
    float *partial_out = nullptr;
    if (bin.kind == kKindHubPieces) {
        const int64_t piece = wave_in_bin;  // G == 64: one piece per wavefront
        if (piece < bin.n_items) {
            if (a.p_chunks) {
                const int64_t *p = a.p_chunks + 4 * (bin.item_begin + piece);
                row = p[0]; e0 = p[1]; e1 = p[2]; wdelta = p[3];
            } else {
                const int64_t *p = a.chunks + 3 * (bin.item_begin + piece);
                row = p[0]; e0 = p[1]; e1 = p[2];
            }
            partial_out = a.partial + (bin.item_begin + piece) * a.ldp;
        }
    } else {
        const int64_t item = wave_in_bin * (64 >> bin.log2_g) + (lane >> bin.log2_g);
        if (item < bin.n_items) {
            row = a.row_perm ? int64_t(a.row_perm[bin.item_begin + item]) : bin.item_begin + item;
            if (a.p_indptr) {
                e0 = a.p_indptr[bin.item_begin + item];
                e1 = a.p_indptr[bin.item_begin + item + 1];
                if (COEF) wdelta = load_ip(a.indptr, a.ip64, row) - e0;
            } else {
                e0 = load_ip(a.indptr, a.ip64, row);
                e1 = load_ip(a.indptr, a.ip64, row + 1);
            }
            row_len = e1 - e0;
        }
    }

    float acc[NPASS][VEC];
#pragma unroll
    for (int p = 0; p < NPASS; ++p)
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[p][i] = 0.0f;

    // the slice that holds the last, short line of the rows gathers it from the dense tail table
    const bool is_tail = slice == a.tail_slice;
    const bool own_table = is_tail || a.slice_stride > 0;  // columns are addressed within the slice
    const T *__restrict__ X = is_tail ? static_cast<const T *>(a.X_tail)
                                      : static_cast<const T *>(a.X) + int64_t(slice) * a.slice_stride;
    const int64_t ldx = is_tail ? a.ld_tail : (a.slice_stride > 0 ? int64_t(a.slice_cols) : a.ldx);
    int col[NPASS];    // column in the output (and in a caller's matrix)
    int lcol[NPASS];   // column in the table this slice gathers from
    int ncols[NPASS];  // valid columns of the strip (< VEC only for the last strip of a padded matrix)
    bool col_ok[NPASS];
#pragma unroll
    for (int p = 0; p < NPASS; ++p) {
        const int lc = (p * C + c) * VEC;
        col[p] = col_base + lc;
        lcol[p] = own_table ? lc : col[p];
        col_ok[p] = lc < Fk;
        ncols[p] = Fk - lc < VEC ? Fk - lc : VEC;
    }

    // Neighbour ids (and coefficients) travel in coalesced tiles of G edges per group; the next tiles
    // are requested before the current ones are consumed, so only the first index loads of a row are
    // exposed latency.  The one-strip fp32 kernel (the sliced launches) asks for two tiles at a time: the
    // lines of the index stream that a row spans are then touched once instead of once per tile, with
    // some thousand gathers of the compute unit in between (worth 1 %; the other variants would pay for
    // the registers with a wavefront of occupancy).
    constexpr int Q = (sizeof(T) == 4 && NPASS == 1) ? 2 : 1;
    auto fetch_tiles = [&](int64_t e_first, int (&u_out)[Q], float (&cf_out)[Q]) {
#pragma unroll
        for (int q = 0; q < Q; ++q) {
            const int64_t e = e_first + q * G;
            u_out[q] = 0;
            cf_out[q] = 0.0f;
            if (e < e1) {
                u_out[q] = a.indices[e];
                if (COEF) {
                    cf_out[q] = a.w ? a.w[e + wdelta] : 1.0f;
                    if (a.edge_scale) cf_out[q] *= a.edge_scale[e + wdelta];
                }
            }
        }
    };
    int nxt_u[Q];
    float nxt_cf[Q];
    fetch_tiles(e0 + lane_in_g, nxt_u, nxt_cf);
    for (int64_t first = e0; __any(first < e1); first += Q * G) {
    int cur_u[Q];
    float cur_cf[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) { cur_u[q] = nxt_u[q]; cur_cf[q] = nxt_cf[q]; }
    fetch_tiles(first + Q * G + lane_in_g, nxt_u, nxt_cf);
#pragma unroll 1
    for (int q = 0; q < Q; ++q) {
        const int64_t tile = first + q * G;
        if (Q > 1 && !__any(tile < e1)) break;
        const int my_u = cur_u[0];
        const float my_cf = cur_cf[0];
#pragma unroll
        for (int i = 0; i + 1 < Q; ++i) { cur_u[i] = cur_u[i + 1]; cur_cf[i] = cur_cf[i + 1]; }
        const int64_t left = e1 - tile;
        const int n_tile = left < G ? (left > 0 ? int(left) : 0) : G;

        for (int j0 = 0; __any(j0 < n_tile); j0 += SR * U) {
            int u[U];
            float cf[U];
            bool ok[U];
#pragma unroll
            for (int k = 0; k < U; ++k) {
                const int j = j0 + k * SR + s;
                const int src_lane = gbase + (j & (G - 1));
                u[k] = __shfl(my_u, src_lane);
                if (COEF) cf[k] = __shfl(my_cf, src_lane);
                ok[k] = j < n_tile;
            }
            // bf16 strips stay packed until they are added (see Strip); fp32 strips are floats already,
            // and the plain arrays schedule slightly better (F=256: 12.04 against 12.26 ms)
            constexpr bool PACKED = sizeof(T) == 2;
            typename Strip<T, VEC>::raw_t xr_[PACKED ? U : 1][NPASS];
            float x[PACKED ? 1 : U][NPASS][VEC];
#pragma unroll
            for (int k = 0; k < U; ++k) {
                // Bit 31 of an index marks a rarely gathered ("cold") source (plan-owned index copy):
                // its row is fetched with a non-temporal load, so that it does not displace the
                // warm rows of the L2.
                const int32_t src = u[k] & 0x7FFFFFFF;
                const bool cold = a.cold_on && (u[k] < 0 || src >= a.warm_rank);
                const T *xr = X + int64_t(src) * ldx;
#pragma unroll
                for (int p = 0; p < NPASS; ++p) {
                    if (ok[k] && col_ok[p]) {
                        if constexpr (PACKED) {
                            if (cold) xr_[k][p] = Strip<T, VEC>::load_nt(xr + lcol[p]);
                            else xr_[k][p] = Strip<T, VEC>::load(xr + lcol[p]);
                        } else {
                            if (cold) VecIO<T, VEC>::load_nt(xr + lcol[p], x[k][p]);
                            else VecIO<T, VEC>::load(xr + lcol[p], x[k][p]);
                        }
                    } else {
                        if constexpr (PACKED) {
                            xr_[k][p] = Strip<T, VEC>::zero();
                        } else {
#pragma unroll
                            for (int i = 0; i < VEC; ++i) x[k][p][i] = 0.0f;
                        }
                    }
                }
            }
#pragma unroll
            for (int k = 0; k < U; ++k)
#pragma unroll
                for (int p = 0; p < NPASS; ++p) {
                    float xv[VEC];
                    if constexpr (PACKED) {
                        Strip<T, VEC>::unpack(xr_[k][p], xv);
                    } else {
#pragma unroll
                        for (int i = 0; i < VEC; ++i) xv[i] = x[k][p][i];
                    }
#pragma unroll
                    for (int i = 0; i < VEC; ++i) {
                        if (COEF) acc[p][i] = fmaf(ok[k] ? cf[k] : 0.0f, xv[i], acc[p][i]);
                        else acc[p][i] += xv[i];
                    }
                }
        }
    }
    }

    // combine the edge slots of the group
    for (int off = C; off < G; off <<= 1) {
#pragma unroll
        for (int p = 0; p < NPASS; ++p)
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[p][i] += __shfl_xor(acc[p][i], off);
    }

    if (row < 0 || s != 0) return;
    if (bin.kind == kKindHubPieces) {
#pragma unroll
        for (int p = 0; p < NPASS; ++p)
            if (col_ok[p]) store_f32<VEC>(partial_out + col[p], acc[p]);
        return;
    }
    const float ds = scale_of(a.dst_mode, row_len);
    const int64_t self_row = (a.self_mode != kSelfNone && a.row_map) ? int64_t(a.row_map[row]) : row;
    const float self_cf = a.self_mode == kSelfInvPlus1 ? scale_of(kScaleInvPlus1, a.col_counts[row]) : 1.0f;
    T *__restrict__ y = static_cast<T *>(a.Y) + row * a.ldy;
#pragma unroll
    for (int p = 0; p < NPASS; ++p) {
        if (!col_ok[p]) continue;
        if (a.self_mode != kSelfNone) {  // Section 6.1: the vertex's own vector joins the sum
            float xs[VEC];
            VecIO<T, VEC>::load(X + self_row * ldx + lcol[p], xs);
#pragma unroll
            for (int i = 0; i < VEC; ++i) acc[p][i] = fmaf(self_cf, xs[i], acc[p][i]);
        }
        float o[VEC];
#pragma unroll
        for (int i = 0; i < VEC; ++i) o[i] = acc[p][i] * ds;
        if (a.bias) {
#pragma unroll
            for (int i = 0; i < VEC; ++i)
                if (i < ncols[p]) o[i] += a.bias[col[p] + i];
        }
        if (a.relu) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) o[i] = o[i] > 0.0f ? o[i] : 0.0f;
        }
        store_strip<T, VEC>(y + col[p], o, ncols[p], a.store_vec);
    }
}

// Adds the pieces of each hub row in their fixed order and writes the row.
template <typename T>
__global__ void __launch_bounds__(256) hub_finalize_kernel(const int32_t *__restrict__ hub_rows, int64_t n_hub,
                                                           const int64_t *__restrict__ piece_offsets,
                                                           const float *__restrict__ partial, const void *indptr,
                                                           int ip64, int dst_mode, T *__restrict__ Y, int64_t ldy,
                                                           int F, int64_t ldp, int self_mode, const OwnRowSrc own,
                                                           const int32_t *__restrict__ col_counts,
                                                           const float *__restrict__ bias, int relu, int col_begin) {
    const int64_t i = blockIdx.x;
    if (i >= n_hub) return;
    const int64_t row = hub_rows[i];
    const int64_t p0 = piece_offsets[i], p1 = piece_offsets[i + 1];
    const float ds = scale_of(dst_mode, load_ip(indptr, ip64, row + 1) - load_ip(indptr, ip64, row));
    for (int colx = col_begin + threadIdx.x; colx < F; colx += blockDim.x) {
        float sum = 0.0f;
        for (int64_t p = p0; p < p1; ++p) sum += partial[p * ldp + colx];
        if (self_mode != kSelfNone)
            sum = fmaf(self_mode == kSelfInvPlus1 ? scale_of(kScaleInvPlus1, col_counts[row]) : 1.0f,
                       own_row_value<T>(own, row, colx), sum);
        float o[1] = {sum * ds};
        if (bias) o[0] += bias[colx];
        if (relu) o[0] = o[0] > 0.0f ? o[0] : 0.0f;
        VecIO<T, 1>::store(Y + row * ldy + colx, o);
    }
}

// ---- source-blocked pieces of the long rows (see blocked.hip) ----
// Four consecutive elements of a per-edge stream, loaded at the alignment of one element.
template <typename E>
struct __attribute__((packed, aligned(alignof(E)))) Packed { E e[4]; };

struct PieceArgs {
    const int32_t *pieces;   // [n_pieces * 4] (begin, length, partial slot, row index)
    int64_t n_pieces;
    const int32_t *idx;      // source ranks, block-major piece order
    const uint16_t *idx16;   // the same as offsets from the block's first rank (null: none); not for the last block
    const uint16_t *piece_block;  // [n_pieces] block of each piece
    int32_t n_blocks, hot_lines, block_lines;
    const uint32_t *epos;    // CSR position of each edge (for the caller's per-edge streams)
    const float *w;          // the caller's weights, read at epos (a random 4-byte read per edge) ...
    const float *w_blk;      // ... or their plan-owned copy in the order of idx (weights bound to the plan)
    const float *scale_blk;  // plan-owned factor of the gathered vertex per edge, in the order of idx
    const void *X;           // first slice table of the launch
    int64_t slice_stride;    // elements between two slice tables
    float *partial;          // [slices][n_pieces][floats per line]
    int32_t log2_slices;
};

// Eight lanes own one piece and one 128-byte line of every gathered row (16 bytes each); a wavefront
// works on eight consecutive pieces, i.e. on 64 lines in flight.  The pieces of a launch follow the
// block order of the layout, so the workgroups that run side by side gather from the same block of
// source rows.  Every piece writes one fp32 partial line; blk_finalize_kernel adds them.
template <typename T, bool COEF>
__global__ void __launch_bounds__(kBlockThreads) piece_kernel(const PieceArgs a) {
    constexpr int VEC = 16 / int(sizeof(T));   // elements per lane
    constexpr int LINE = 8 * VEC;              // elements per line = floats per partial line
    constexpr int U = 8;
    const int lane = threadIdx.x & 63;
    const int slice = int(blockIdx.x) & ((1 << a.log2_slices) - 1);
    const int64_t vblock = int64_t(blockIdx.x) >> a.log2_slices;
    const int c = lane & 7, gbase = lane & ~7;
    const int64_t piece = (vblock * kWavesPerBlock + (threadIdx.x >> 6)) * 8 + (lane >> 3);
    uint32_t begin = 0;
    int len = 0;
    int64_t slot = 0;
    if (piece < a.n_pieces) {
        const int4 d = *reinterpret_cast<const int4 *>(a.pieces + 4 * piece);
        begin = uint32_t(d.x); len = d.y; slot = d.z;
    }
    // the piece's block and its first rank, for the 16-bit indices
    bool narrow = false;
    int base = 0;
    if (a.idx16 && len > 0) {
        const int k = a.piece_block[piece];
        narrow = k < a.n_blocks - 1;
        base = k == 0 ? 0 : a.hot_lines + (k - 1) * a.block_lines;
    }
    const T *__restrict__ X = static_cast<const T *>(a.X) + int64_t(slice) * a.slice_stride + c * VEC;
    float acc[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = 0.0f;

    // The per-edge streams are read a window of 32 edges at a time: lane c of the group holds edges
    // [t + 4c, t + 4c + 4) of the piece, one 8- or 16-byte load per stream (at the 2- or 4-byte
    // alignment of the element: a piece begins anywhere), so a group touches each line of a stream once
    // instead of once per eight edges.  The loads of a lane may run up to three elements past the piece's
    // end (into the next piece, or into the padding behind the arrays); those elements are never used.
    auto fetch = [&](int t, int (&u_out)[4], float (&cf_out)[4]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) { u_out[i] = 0; cf_out[i] = 0.0f; }
        const int j = t + 4 * c;
        if (j < len) {
            const uint32_t pos = begin + uint32_t(j);
            if (narrow) {
                Packed<uint16_t> v;
                __builtin_memcpy(&v, a.idx16 + pos, sizeof(v));
#pragma unroll
                for (int i = 0; i < 4; ++i) u_out[i] = base + int(v.e[i]);
            } else {
                Packed<int32_t> v;
                __builtin_memcpy(&v, a.idx + pos, sizeof(v));
#pragma unroll
                for (int i = 0; i < 4; ++i) u_out[i] = v.e[i];
            }
            if (COEF) {
#pragma unroll
                for (int i = 0; i < 4; ++i) cf_out[i] = 1.0f;
                if (a.w_blk) {
                    Packed<float> v;
                    __builtin_memcpy(&v, a.w_blk + pos, sizeof(v));
#pragma unroll
                    for (int i = 0; i < 4; ++i) cf_out[i] = v.e[i];
                } else if (a.w) {
                    Packed<uint32_t> v;
                    __builtin_memcpy(&v, a.epos + pos, sizeof(v));
#pragma unroll
                    for (int i = 0; i < 4; ++i) cf_out[i] = j + i < len ? a.w[v.e[i]] : 0.0f;
                }
                if (a.scale_blk) {
                    Packed<float> v;
                    __builtin_memcpy(&v, a.scale_blk + pos, sizeof(v));
#pragma unroll
                    for (int i = 0; i < 4; ++i) cf_out[i] *= v.e[i];
                }
            }
        }
    };
    int nxt_u[4];
    float nxt_cf[4];
    fetch(0, nxt_u, nxt_cf);
    for (int t0 = 0; __any(t0 < len); t0 += 32) {
        int my_u[4];
        float my_cf[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { my_u[i] = nxt_u[i]; my_cf[i] = nxt_cf[i]; }
        fetch(t0 + 32, nxt_u, nxt_cf);
        for (int m = 0; m < 4; ++m) {
            const int t = t0 + U * m;
            if (!__any(t < len)) break;
            typename Strip<T, VEC>::raw_t x[U];
            float cf[U];
#pragma unroll
            for (int k = 0; k < U; ++k) {
                const int src = gbase + 2 * m + (k >> 2);
                const int u = __shfl(my_u[k & 3], src);
                if (COEF) cf[k] = __shfl(my_cf[k & 3], src);
                if (t + k < len) x[k] = Strip<T, VEC>::load(X + int64_t(u) * LINE);
                else x[k] = Strip<T, VEC>::zero();
            }
#pragma unroll
            for (int k = 0; k < U; ++k) {
                float xv[VEC];
                Strip<T, VEC>::unpack(x[k], xv);
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    if (COEF) acc[i] = fmaf(t + k < len ? cf[k] : 0.0f, xv[i], acc[i]);
                    else acc[i] += xv[i];
                }
            }
        }
    }
    if (piece < a.n_pieces) {
        float *out = a.partial + (int64_t(slice) * a.n_pieces + slot) * LINE + c * VEC;
#pragma unroll
        for (int i = 0; i < VEC; i += 4) {
            const f32x4 v = {acc[i], acc[i + 1], acc[i + 2], acc[i + 3]};
            __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(out + i));
        }
    }
}

// Adds the partial lines of every long row in a fixed order and writes the columns [0, fw) of the
// launch.  Eight lanes own one (row, slice) pair, 16 bytes of the output row each, so a wavefront
// finishes eight rows of a slice.  The sums themselves are formed by the whole wavefront, one of its
// eight pairs after the other: lane group g adds the partial lines g, g + 8, g + 16, ... of the pair (a
// wavefront load covers eight consecutive lines, 1 KB), and the eight group sums are added pairwise
// (groups 0+1, 2+3, ... then 0..1 + 2..3, ...).  A hub row has thousands of partial lines: added by its
// own eight lanes alone, one such row set the duration of the launch.
template <typename T>
__global__ void __launch_bounds__(256) blk_finalize_kernel(const int32_t *__restrict__ rows, int64_t n_rows,
                                                           const uint32_t *__restrict__ rowbase,
                                                           const float *__restrict__ partial, int64_t n_pieces, int n_slices,
                                                           const void *indptr, int ip64, int dst_mode, T *__restrict__ Y,
                                                           int64_t ldy, int fw, int store_vec, int self_mode,
                                                           const OwnRowSrc own,
                                                           const int32_t *__restrict__ col_counts,
                                                           const float *__restrict__ bias, int relu) {
    constexpr int VEC = 16 / int(sizeof(T));  // output columns per lane
    constexpr int LINE = 8 * VEC;             // columns per slice = floats per partial line
    const int lane = threadIdx.x & 63;
    const int g = lane >> 3, c = lane & 7;
    const int64_t n_items = n_rows * n_slices;
    const int64_t first_item = ((int64_t(blockIdx.x) * blockDim.x + threadIdx.x) >> 6) << 3;  // wave-uniform
    if (first_item >= n_items) return;
    float mine[VEC];  // the sum of this group's own pair
#pragma unroll
    for (int k = 0; k < VEC; ++k) mine[k] = 0.0f;
    for (int j = 0; j < 8; ++j) {
        const int64_t item = first_item + j;
        if (item >= n_items) break;
        const int64_t i = item % n_rows;
        const int slice = int(item / n_rows);
        const int64_t p0 = rowbase[i], p1 = rowbase[i + 1];
        const float *__restrict__ src = partial + int64_t(slice) * n_pieces * LINE + c * VEC;
        float sum[VEC];
#pragma unroll
        for (int k = 0; k < VEC; ++k) sum[k] = 0.0f;
        auto load_line = [&](int64_t p, f32x4 (&v)[VEC / 4]) {
#pragma unroll
            for (int q = 0; q < VEC / 4; ++q) {
                v[q] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
                if (p < p1) v[q] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(src + p * LINE) + q);
            }
        };
        auto add_line = [&](const f32x4 (&v)[VEC / 4]) {
#pragma unroll
            for (int q = 0; q < VEC / 4; ++q) {
                sum[4 * q] += v[q].x; sum[4 * q + 1] += v[q].y; sum[4 * q + 2] += v[q].z; sum[4 * q + 3] += v[q].w;
            }
        };
        for (int64_t p = p0 + g; p < p1; p += 32) {  // four lines per group in flight
            f32x4 v0[VEC / 4], v1[VEC / 4], v2[VEC / 4], v3[VEC / 4];
            load_line(p, v0); load_line(p + 8, v1); load_line(p + 16, v2); load_line(p + 24, v3);
            add_line(v0); add_line(v1); add_line(v2); add_line(v3);
        }
#pragma unroll
        for (int off = 8; off < 64; off <<= 1)
#pragma unroll
            for (int k = 0; k < VEC; ++k) sum[k] += __shfl_xor(sum[k], off);
        if (g == j) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) mine[k] = sum[k];
        }
    }
    const int64_t item = first_item + g;
    if (item >= n_items) return;
    const int64_t i = item % n_rows;
    const int slice = int(item / n_rows);
    const int col0 = slice * LINE + c * VEC;
    if (col0 >= fw) return;
    const int64_t row = rows[i];
    const int ncols = fw - col0 < VEC ? fw - col0 : VEC;
    const float ds = scale_of(dst_mode, load_ip(indptr, ip64, row + 1) - load_ip(indptr, ip64, row));
    const float self_cf = self_mode == kSelfInvPlus1 ? scale_of(kScaleInvPlus1, col_counts[row]) : 1.0f;
    float o[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) {
        float v = mine[k];
        if (k < ncols) {
            if (self_mode != kSelfNone) v = fmaf(self_cf, own_row_value<T>(own, row, col0 + k), v);
            v *= ds;
            if (bias) v += bias[col0 + k];
            if (relu) v = v > 0.0f ? v : 0.0f;
        }
        o[k] = v;
    }
    store_strip<T, VEC>(Y + row * ldy + col0, o, ncols, store_vec);
}

// Copies the gathered matrix into rows of whole 128-byte lines (plan-owned buffer), so that
// 16-byte loads and XCD column slices apply to widths like 100 or 602.  One thread per chunk of
// sizeof(V) bytes; V is the widest type the source rows allow.
template <typename V>
__global__ void __launch_bounds__(256) pad_rows_kernel(const V *__restrict__ src, int64_t ld_src, V *__restrict__ dst,
                                                       int64_t ld_dst, int64_t N, int chunks_per_row,
                                                       const int32_t *__restrict__ row_map, int log2_chunks_per_line,
                                                       int64_t table_stride, int log2_tpr) {
    // 2^log2_tpr consecutive threads walk the chunks of one row (no division per chunk)
    const int tpr = 1 << log2_tpr;
    const int64_t rows_per_block = blockDim.x >> log2_tpr;
    const int c0 = threadIdx.x & (tpr - 1);
    for (int64_t row = int64_t(blockIdx.x) * rows_per_block + (threadIdx.x >> log2_tpr); row < N;
         row += int64_t(gridDim.x) * rows_per_block) {
        const int64_t drow = row_map ? int64_t(row_map[row]) : row;
        const V *in = src + row * ld_src;
        for (int c = c0; c < chunks_per_row; c += tpr) {
            // row-major: log2_chunks_per_line is 31 (one table); slice-major: one table per line
            const int line = c >> log2_chunks_per_line, within = c - (line << log2_chunks_per_line);
            // 16-byte chunks go out non-temporal; smaller ones as plain stores, which the L2 merges into lines
            V *q = &dst[line * table_stride + drow * ld_dst + within];
            if constexpr (sizeof(V) >= 16) __builtin_nontemporal_store(in[c], q);
            else *q = in[c];
        }
    }
}

// Same copy for fp32 rows, with row v multiplied by the factor its vertex carries as a gathered
// row (1/din, 1/sqrt(deg) or 1/(din+1)): folding the factor into the copy that happens anyway
// saves the per-edge factor stream and the per-edge multiply of MEAN / SAGE_GCN backward and GCN.
template <int W>
__global__ void __launch_bounds__(256) pad_scale_rows_kernel(const float *__restrict__ src, int64_t ld_src,
                                                             float *__restrict__ dst, int64_t ld_dst, int64_t N,
                                                             int chunks_per_row, int mode,
                                                             const int32_t *__restrict__ counts,
                                                             const int32_t *__restrict__ row_map, int log2_chunks_per_line,
                                                             int64_t table_stride, int log2_tpr) {
    const int tpr = 1 << log2_tpr;
    const int64_t rows_per_block = blockDim.x >> log2_tpr;
    const int c0 = threadIdx.x & (tpr - 1);
    for (int64_t row = int64_t(blockIdx.x) * rows_per_block + (threadIdx.x >> log2_tpr); row < N;
         row += int64_t(gridDim.x) * rows_per_block) {
        const float f = scale_of(mode, counts[row]);
        const int64_t drow = row_map ? int64_t(row_map[row]) : row;
        const float *in = src + row * ld_src;
        for (int c = c0; c < chunks_per_row; c += tpr) {
            float v[W];
            VecIO<float, W>::load(in + int64_t(c) * W, v);
#pragma unroll
            for (int i = 0; i < W; ++i) v[i] *= f;
            const int line = c >> log2_chunks_per_line, within = c - (line << log2_chunks_per_line);
            float *q = dst + line * table_stride + drow * ld_dst + int64_t(within) * W;
            if constexpr (W == 4) {
                VecIO<float, 4>::store(q, v);
            } else {
#pragma unroll
                for (int i = 0; i < W; ++i) q[i] = v[i];
            }
        }
    }
}

// Threads per row of the pad kernels (a power of two <= 256 covering the row's chunks) and the grid.
static inline void pad_launch_shape(int64_t N, int cpr, int *log2_tpr, unsigned *blocks) {
    // the power of two (>= 8 threads: one 128-byte line of 16-byte chunks) that leaves the fewest idle
    // slots in the last round over the row's chunks; the widest among equals
    int l = 0;
    int64_t best_waste = INT64_MAX;
    for (int cand = 8; cand >= 3; --cand) {
        const int64_t tpr = int64_t(1) << cand;
        const int64_t waste = (cpr + tpr - 1) / tpr * tpr - cpr;
        if (waste < best_waste) { best_waste = waste; l = cand; }
    }
    if (cpr < 8) { l = 0; while ((1 << l) < cpr) ++l; }
    *log2_tpr = l;
    const int64_t rows_per_block = 256 >> l;
    int64_t b = (N + rows_per_block - 1) / rows_per_block;
    if (b > (int64_t(1) << 17)) b = int64_t(1) << 17;
    *blocks = static_cast<unsigned>(b > 0 ? b : 1);
}

template <int W>
hipError_t launch_pad_scale(const void *src, int64_t ld_src, void *dst, int64_t ld_dst, int64_t N, int64_t F, int mode,
                            const int32_t *counts, hipStream_t stream, const int32_t *row_map = nullptr,
                            int64_t table_stride = 0) {
    const int cpr = int(F / W);
    int log2_tpr;
    unsigned blocks;
    pad_launch_shape(N, cpr, &log2_tpr, &blocks);
    pad_scale_rows_kernel<W><<<blocks, 256, 0, stream>>>(
        static_cast<const float *>(src), ld_src, static_cast<float *>(dst), ld_dst, N, cpr, mode, counts, row_map,
        table_stride > 0 ? gnn_ilog2_ceil(32 / W) : 31, table_stride, log2_tpr);
    return hipGetLastError();
}

template <typename V>
hipError_t launch_pad(const void *src, int64_t ld_src_bytes, void *dst, int64_t ld_dst_bytes, int64_t N,
                      int64_t row_bytes, hipStream_t stream, const int32_t *row_map = nullptr,
                      int64_t table_stride_bytes = 0) {
    const int cpr = int(row_bytes / sizeof(V));
    int log2_tpr;
    unsigned blocks;
    pad_launch_shape(N, cpr, &log2_tpr, &blocks);
    pad_rows_kernel<V><<<blocks, 256, 0, stream>>>(
        static_cast<const V *>(src), ld_src_bytes / int64_t(sizeof(V)), static_cast<V *>(dst),
        ld_dst_bytes / int64_t(sizeof(V)), N, cpr, row_map,
        table_stride_bytes > 0 ? gnn_ilog2_ceil(int64_t(128 / sizeof(V))) : 31, table_stride_bytes / int64_t(sizeof(V)), log2_tpr);
    return hipGetLastError();
}

// ---------------------------------------------------------------- host side
template <typename T, int VEC, bool COEF>
hipError_t launch_npass(int npass, dim3 grid, hipStream_t stream, const AggArgs &a) {
    switch (npass) {
        case 1: aggregate_kernel<T, VEC, 1, COEF><<<grid, kBlockThreads, 0, stream>>>(a); break;
        case 2: aggregate_kernel<T, VEC, 2, COEF><<<grid, kBlockThreads, 0, stream>>>(a); break;
        case 3: aggregate_kernel<T, VEC, 3, COEF><<<grid, kBlockThreads, 0, stream>>>(a); break;
        case 4: aggregate_kernel<T, VEC, 4, COEF><<<grid, kBlockThreads, 0, stream>>>(a); break;
        case 5: aggregate_kernel<T, VEC, 5, COEF><<<grid, kBlockThreads, 0, stream>>>(a); break;
        case 6: aggregate_kernel<T, VEC, 6, COEF><<<grid, kBlockThreads, 0, stream>>>(a); break;
        default: aggregate_kernel<T, VEC, 8, COEF><<<grid, kBlockThreads, 0, stream>>>(a); break;
    }
    return hipGetLastError();
}

template <typename T, int VEC>
hipError_t launch_coef(bool coef, int npass, dim3 grid, hipStream_t stream, const AggArgs &a) {
    return coef ? launch_npass<T, VEC, true>(npass, grid, stream, a) : launch_npass<T, VEC, false>(npass, grid, stream, a);
}

constexpr int kMaxPass = 8;

// A library-owned second stream per device (default priority, created on first use, kept until the process
// ends): the launches over the short rows run there while the caller's stream sweeps the source blocks of the
// long rows.
hipStream_t overlap_stream() {
    static std::mutex mu;
    static hipStream_t streams[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!streams[dev] && hipStreamCreateWithFlags(&streams[dev], hipStreamNonBlocking) != hipSuccess) streams[dev] = nullptr;
    return streams[dev];
}

// One direction of the aggregation.  `gathered` is X (forward) or dY (backward).  bias / relu:
// the epilogue of a fused layer (out = act(aggregate + bias)), or nullptr / 0.
// no_alloc: the hub partial sums go into the library's fixed device array and the call allocates
// nothing (gnn_aggregate_fwd_noalloc); else into the plan's or the caller's workspace.
int run_aggregate(const void *indptr, const int32_t *indices, const float *w, const void *gathered, void *out,
                  int64_t N, int64_t F, int op, const gnn_opts *opts_in, bool backward, const float *bias = nullptr,
                  int relu = 0, bool no_alloc = false, bool prepacked = false, void *ext_tables = nullptr,
                  int64_t ext_bytes = 0, bool pack_only = false) {
    // prepacked: the gathered matrix already lies in the plan's layout (written there by a producer, see
    // gnn_packed_target_for, or by an earlier pack_only call); `gathered` is not read, no copy is made.
    // ext_tables: that layout lives in the caller's buffer of ext_bytes instead of the plan's.
    // pack_only: write the layout from `gathered` and return.
    gnn_opts o{};
    if (opts_in) o = *opts_in;
    if (no_alloc) {
        // nothing that a plan would have to grow: rows are gathered where they lie, from the caller's index array
        o.flags = (o.flags | GNN_FLAG_NO_PADDED_COPY | GNN_FLAG_NO_COLD_HINTS) &
                  ~(GNN_FLAG_FORCE_PADDED_COPY | GNN_FLAG_FORCE_COLD_HINTS);
        o.workspace = nullptr;
        o.workspace_bytes = 0;
    }
    if (N < 0 || F < 0) return GNN_ERR_INVALID_ARG;
    if (op != GNN_SUM && op != GNN_MEAN && op != GNN_GCN_SYM && op != GNN_SAGE_GCN) return GNN_ERR_INVALID_ARG;
    if (o.dtype != GNN_F32 && o.dtype != GNN_BF16) return GNN_ERR_INVALID_ARG;
    if (o.max_slices != 0 && o.max_slices != 1 && o.max_slices != 2 && o.max_slices != 4 && o.max_slices != 8)
        return GNN_ERR_INVALID_ARG;
    if (N == 0 || F == 0) return GNN_OK;
    if (!indptr || (!gathered && !prepacked) || !out) return GNN_ERR_INVALID_ARG;
    if (N > INT32_MAX || F > INT32_MAX) return GNN_ERR_INVALID_ARG;
    if ((prepacked || pack_only) && !o.plan) return GNN_ERR_UNSUPPORTED;
    if (prepacked && !ext_tables && (o.dtype != GNN_F32 || w)) return GNN_ERR_INVALID_ARG;
    if (prepacked && pack_only) return GNN_ERR_INVALID_ARG;
    if (prepacked) { gathered = nullptr; o.ldx = 0; }
    const int64_t ldx = o.ldx ? o.ldx : F, ldy = o.ldy ? o.ldy : F;
    if (ldx < F || ldy < F) return GNN_ERR_INVALID_ARG;
    gnn_plan *plan = o.plan;
    if (plan && (plan->n_rows != N || plan->indptr_is_64 != (o.indptr_is_64 ? 1 : 0))) return GNN_ERR_INVALID_ARG;
    if (plan && plan->n_edges > 0 && !indices) return GNN_ERR_INVALID_ARG;

    // scaling of the edge terms and of the output row
    int src_mode = kScaleNone, dst_mode = kScaleNone;
    if (op == GNN_MEAN) {
        if (backward) src_mode = kScaleInv; else dst_mode = kScaleInv;
    } else if (op == GNN_GCN_SYM && !w) {
        src_mode = kScaleRsqrt;
        dst_mode = kScaleRsqrt;
    }
    int self_mode = kSelfNone;
    if (op == GNN_SAGE_GCN) {  // (sum + own vector) / (din + 1) and its adjoint
        if (backward) { src_mode = kScaleInvPlus1; self_mode = kSelfInvPlus1; }
        else { dst_mode = kScaleInvPlus1; self_mode = kSelfPlain; }
    }
    if ((src_mode != kScaleNone || self_mode == kSelfInvPlus1) && !plan) return GNN_ERR_UNSUPPORTED;  // needs the column counts a plan holds
    const float *edge_scale = nullptr;

    const int esz = o.dtype == GNN_BF16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(gathered) % esz || reinterpret_cast<uintptr_t>(out) % esz) return GNN_ERR_INVALID_ARG;
    const int max_vec = 16 / esz;
    const int64_t line_elems = 128 / esz;

    hipStream_t stream = static_cast<hipStream_t>(o.stream);
    (void)hipGetLastError();  // a stale error of an earlier, failed call must not be blamed on this one

    // Gathered rows that are not whole 128-byte lines (F = 100, 602, or a misaligned base) are
    // first copied into a plan-owned matrix of padded rows: one streaming pass over N*F elements,
    // small next to the E*F gather, buys 16-byte loads and the XCD column slices below.
    int64_t ldg = ldx;  // row stride of the matrix the kernel gathers from
    bool padded = false;
    // explicit weights keep a plan that blocks by itself on the path without pieces unless they are bound to it
    const bool blocks_expected = plan && !(o.flags & GNN_FLAG_NO_SOURCE_BLOCKS) && gnn_plan_blocks_expected(plan, int(esz)) &&
                                 (!w || w == plan->bound_w || plan->blocking.min_degree > 0);
    const gnn_layout layout = gnn_choose_layout(plan, N, F, esz, ldx, reinterpret_cast<uintptr_t>(gathered) % 128 == 0,
                                                o.flags, o.max_slices, /*allow_tail=*/o.max_slices != 1,
                                                /*scaled_source=*/src_mode != kScaleNone, blocks_expected);
    // what a producer can write into: the slice tables in rank order (the layout gnn_packed_target_for describes)
    if ((prepacked || pack_only) &&
        !(layout.padded_copy && layout.slice_major && !(o.flags & GNN_FLAG_NO_RANK_ORDER) && plan->n_edges > 0))
        return ext_tables ? GNN_ERR_UNSUPPORTED : GNN_ERR_INVALID_ARG;
    const bool slices_wanted = layout.slices_wanted;
    // the caller's matrix stays the source of the own-row term of the hub rows (hub_finalize_kernel)
    const void *orig = gathered;
    const int orig_self_mode = self_mode;
    const char *tail_table = nullptr;
    bool slice_major = false;  // the copy holds one table per 128-byte column slice
    gnn_rank_layout rl{};  // rank layout of the copy (see gnn_plan)
    const int32_t *rank = nullptr, *rank_indices = nullptr;
    void *tables = nullptr;  // the copy: the plan's buffer or the caller's
    bool factor_in_tables = false;
    if (layout.padded_copy) {
        int rc = GNN_OK;
        if (ext_tables) {
            if (ext_bytes < layout.bytes || reinterpret_cast<uintptr_t>(ext_tables) % 128) return GNN_ERR_INVALID_ARG;
            tables = ext_tables;
        } else {
            rc = gnn_plan_padded(plan, layout.bytes);
            if (rc != GNN_OK) return rc;
            tables = plan->padded;
        }
        if (!(o.flags & GNN_FLAG_NO_RANK_ORDER) && plan->n_edges > 0) {
            rc = gnn_plan_rank_indices(plan, indptr, indices, (o.flags & GNN_FLAG_FORCE_COLD_HINTS) != 0, stream, &rl);
            if (rc != GNN_OK) return rc;
            rank = rl.rank;
            rank_indices = rl.indices;
        }
        const bool scale_in_copy = esz == 4 && src_mode != kScaleNone;  // fp32: the factor of the gathered rows goes into the copy
        factor_in_tables = scale_in_copy;
        if ((prepacked || pack_only) && !rank) return GNN_ERR_UNSUPPORTED;
        const int copy_mode = src_mode;
        // copies `ncols` columns starting at `src` into rows of stride dst_ld, with the widest chunks the source allows
        auto copy_part = [&](const char *src, int64_t ncols, char *dst, int64_t dst_ld, int64_t tstride) -> hipError_t {
            const int64_t row_bytes = ncols * esz, src_ld_bytes = ldx * esz, dst_ld_bytes = dst_ld * esz;
            const uintptr_t addr = reinterpret_cast<uintptr_t>(src);
            if (scale_in_copy) {
                if (row_bytes % 16 == 0 && src_ld_bytes % 16 == 0 && addr % 16 == 0)
                    return launch_pad_scale<4>(src, ldx, dst, dst_ld, N, ncols, copy_mode, plan->col_counts, stream, rank, tstride);
                if (row_bytes % 8 == 0 && src_ld_bytes % 8 == 0 && addr % 8 == 0)
                    return launch_pad_scale<2>(src, ldx, dst, dst_ld, N, ncols, copy_mode, plan->col_counts, stream, rank, tstride);
                return launch_pad_scale<1>(src, ldx, dst, dst_ld, N, ncols, copy_mode, plan->col_counts, stream, rank, tstride);
            }
            if (row_bytes % 16 == 0 && src_ld_bytes % 16 == 0 && addr % 16 == 0)
                return launch_pad<u32x4>(src, src_ld_bytes, dst, dst_ld_bytes, N, row_bytes, stream, rank, tstride * esz);
            if (row_bytes % 8 == 0 && src_ld_bytes % 8 == 0 && addr % 8 == 0)
                return launch_pad<u32x2>(src, src_ld_bytes, dst, dst_ld_bytes, N, row_bytes, stream, rank, tstride * esz);
            if (row_bytes % 4 == 0 && src_ld_bytes % 4 == 0 && addr % 4 == 0)
                return launch_pad<uint32_t>(src, src_ld_bytes, dst, dst_ld_bytes, N, row_bytes, stream, rank, tstride * esz);
            return launch_pad<uint16_t>(src, src_ld_bytes, dst, dst_ld_bytes, N, row_bytes, stream, rank, tstride * esz);
        };
        const int64_t main_cols = F - layout.tail_elems;
        char *dst = static_cast<char *>(tables);
        if (!prepacked &&
            copy_part(static_cast<const char *>(gathered), main_cols, dst, layout.ld_pad, layout.table_stride) != hipSuccess)
            return GNN_ERR_LAUNCH;
        if (layout.tail_elems > 0) {
            // behind the main part, a multiple of 128 bytes into the buffer
            char *tail_dst = dst + (layout.slice_major ? layout.main_lines * layout.table_stride : N * layout.ld_pad) * esz;
            if (!prepacked &&
                copy_part(static_cast<const char *>(gathered) + main_cols * esz, layout.tail_elems, tail_dst, layout.tail_ld, 0) != hipSuccess)
                return GNN_ERR_LAUNCH;
            tail_table = tail_dst;
        }
        if (scale_in_copy) {
            src_mode = kScaleNone;
            if (self_mode == kSelfInvPlus1) self_mode = kSelfPlain;  // the own row is already scaled
        }
        if (pack_only) return GNN_OK;
        gathered = tables;
        ldg = layout.ld_pad;
        padded = true;
        slice_major = layout.slice_major;
    }

    if (src_mode != kScaleNone && plan->n_edges > 0) {
        // streamed per-edge factors (built once per plan and mode) instead of a random 4-byte
        // lookup per edge, which would cost a 128-byte line each
        if (no_alloc && !plan->edge_scale[src_mode - 1]) return GNN_ERR_UNSUPPORTED;  // gnn_plan_prepare builds it
        int rc = gnn_plan_edge_scale(plan, indices, src_mode, stream, &edge_scale);
        if (rc != GNN_OK) return rc;
    }
    const bool coef = (w != nullptr) || src_mode != kScaleNone;

    // Widest load the gathered rows allow.  Only the padded copy may be read past column F (its
    // rows end in padding that belongs to the buffer); a caller's matrix needs F % vec == 0 unless
    // the caller vouches for the padding (GNN_FLAG_PADDED_ROWS).
    int vec = max_vec;
    const bool rows_padded = padded || (o.flags & GNN_FLAG_PADDED_ROWS) != 0;  // then ldg % vec == 0 covers the over-read
    while (vec > 1 && !(ldg % vec == 0 && reinterpret_cast<uintptr_t>(gathered) % (uintptr_t(vec) * esz) == 0 &&
                        (rows_padded || F % vec == 0)))
        vec >>= 1;
    // Widest store the output rows allow (partial strips fall back to single elements).
    int store_vec = vec;
    while (store_vec > 1 && !(ldy % store_vec == 0 && reinterpret_cast<uintptr_t>(out) % (uintptr_t(store_vec) * esz) == 0))
        store_vec >>= 1;

    // hub scratch
    float *partial = nullptr;
    const bool has_hub = plan && plan->n_chunks > 0;
    if (has_hub) {
        const int64_t need = gnn_plan_workspace_bytes(plan, F);
        if (no_alloc) {
            if (need > int64_t(GNN_NOALLOC_SCRATCH_BYTES)) return GNN_ERR_SCRATCH_CAPACITY;
            const int rc = static_scratch_of_current_device(&partial);
            if (rc != GNN_OK) return rc;
        } else if (o.workspace && o.workspace_bytes >= need) {
            partial = static_cast<float *>(o.workspace);
        } else if (o.workspace) {
            return GNN_ERR_INVALID_ARG;
        } else {
            int rc = gnn_plan_reserve(plan, F);
            if (rc != GNN_OK) return rc;
            partial = static_cast<float *>(plan->scratch);
        }
        if (reinterpret_cast<uintptr_t>(partial) % 16) return GNN_ERR_INVALID_ARG;
    }

    // Column slices over the XCDs.  Workgroups are handed to the 8 XCDs round-robin by
    // workgroup id, and every XCD has a private L2.  When the gathered rows are whole 128-byte
    // lines, workgroup b of a launch gathers only column slice (b % S): an XCD's L2 then sees one
    // slice of every gathered row instead of whole rows of an eighth of the destinations, so many
    // more hot source rows stay resident.  Slices are one line wide (wider when the row stride is a
    // multiple of 8 lines: one-line slices would crowd too few L2 channels), and a row of more
    // than 8 slices is covered by several launches of 8, 4, 2 or 1 slices (column slabs in time),
    // so that every launch keeps all 8 XCDs equally busy.  The price is one read of the index
    // stream per slice.
    struct Segment { int64_t f0, fw; int log2_s; int64_t slice_cols; int tail_slice; };
    // Sliced: at most 256 one-unit slices, two or more per launch, plus the tail; unsliced: at most 64 slabs.
    constexpr int kMaxSegs = 130;
    Segment segs[kMaxSegs];
    int n_segs = 0;
    {
        const bool lines_ok = (ldg % line_elems == 0) && reinterpret_cast<uintptr_t>(gathered) % 128 == 0;
        const int64_t lines = (F + line_elems - 1) / line_elems;
        // Slice width: XCD k reads lines {k*w .. k*w+w-1} of rows L lines apart; with L a multiple
        // of 8 (16) a one-line slice would land on 2 (1) of 16 line-interleaved L2 channels, so
        // the slice is widened until it covers at least 4 (measured: L=8, w=2 beats w=1; L=4 and
        // odd L are fastest with w=1).
        int64_t g16 = 1;
        while (g16 < 16 && (ldg / line_elems) % (g16 * 2) == 0) g16 *= 2;
        const int64_t unit_lines = g16 >= 8 ? g16 / 4 : 1;
        const int64_t units = (lines + unit_lines - 1) / unit_lines;
        const int64_t s_max = o.max_slices > 0 ? o.max_slices : 8;
        if (lines_ok && units >= 2 && units <= 256 && s_max >= 2 && slices_wanted) {
            // The last unit is the dense tail, when there is one.  It gets a launch of its own over all
            // XCDs: gathering 16 bytes costs a cache request per edge like a whole line does, and as one
            // slice among others it kept its share of the XCDs busy nearly as long as a full line
            // (F = 100 as 3 + tail in one launch: 5.77 ms; F = 96: 4.52 ms).
            const int64_t main_units = tail_table ? units - 1 : units;
            int64_t u0 = 0;
            while (u0 < main_units) {
                int ls = 3;
                while (ls > 0 && ((int64_t(1) << ls) > main_units - u0 || (int64_t(1) << ls) > s_max)) --ls;
                if (n_segs >= kMaxSegs - 1) return GNN_ERR_UNSUPPORTED;  // rows this wide take the unsliced route (max_slices = 1)
                Segment &g = segs[n_segs++];
                g.f0 = u0 * unit_lines * line_elems;
                g.slice_cols = unit_lines * line_elems;
                g.log2_s = ls;
                const int64_t end = g.f0 + (g.slice_cols << ls);
                g.fw = (end < F ? end : F) - g.f0;
                g.tail_slice = -1;
                u0 += int64_t(1) << ls;
            }
            if (tail_table) {
                Segment &g = segs[n_segs++];
                g.f0 = main_units * unit_lines * line_elems;
                g.slice_cols = layout.tail_ld;  // few column lanes per row group: the lanes go to more edges instead
                g.log2_s = 0;
                g.fw = F - g.f0;
                g.tail_slice = 0;
            }
        } else {
            if (tail_table || slice_major) return GNN_ERR_UNSUPPORTED;  // those layouts are only made for sliced launches
            // no slices: slabs of up to 64 lanes * vec * kMaxPass columns
            const int64_t slab = int64_t(64) * vec * kMaxPass;
            for (int64_t f0 = 0; f0 < F && n_segs < 64; f0 += slab) {
                Segment &g = segs[n_segs++];
                g.f0 = f0;
                g.fw = F - f0 < slab ? F - f0 : slab;
                g.log2_s = 0;
                g.slice_cols = g.fw;
                g.tail_slice = -1;
            }
            if ((F + slab - 1) / slab > 64) return GNN_ERR_UNSUPPORTED;
        }
    }

    // Sliced launches of a large power-law graph gather their rarely used sources with
    // non-temporal loads: the plan keeps a copy of the index array with those sources flagged.
    const int32_t *gather_indices = indices;
    if (rank_indices) {
        gather_indices = rank_indices;  // the copy is in rank order; cold sources are flagged there too
    } else if (plan && ((n_segs > 0 && segs[0].log2_s > 0 && !(o.flags & GNN_FLAG_NO_COLD_HINTS)) ||
                        (o.flags & GNN_FLAG_FORCE_COLD_HINTS))) {
        const int32_t *flagged = nullptr;
        int rc = gnn_plan_cold_indices(plan, indices, (o.flags & GNN_FLAG_FORCE_COLD_HINTS) != 0, stream, &flagged);
        if (rc != GNN_OK) return rc;
        if (flagged) gather_indices = flagged;
    }

    // The long rows of a large power-law graph are served as source-blocked pieces (blocked.hip) in
    // every launch that gathers from slice tables; the dense tail keeps the plain path.
    gnn_blocked_layout bl{};
    const float *scale_blk = nullptr, *w_blk = nullptr;
    if (slice_major && rank_indices && !(o.flags & GNN_FLAG_NO_SOURCE_BLOCKS)) {
        int rc = gnn_plan_blocked(plan, indptr, stream, &bl);
        if (rc != GNN_OK) return rc;
        // Explicit weights sit in CSR order, the pieces in rank order: every edge would cost a random 4-byte
        // read (measured: 1.44 -> 3.67 ms on the weighted workload at F=64), so such calls keep the plain
        // path unless the plan's blocking was asked for explicitly, or the weights were bound to the plan
        // (gnn_plan_bind_edge_weights), which then holds a copy of them in piece order.  The plan's own
        // per-edge factors get such a copy too.
        const bool bound = w && w == plan->bound_w;
        if (bl.active && w && bl.automatic && !bound) bl.active = false;
        // bf16 pieces write partial lines twice as large as the lines they gather: on graphs of a few
        // L2s' worth of vertices that eats the gain (233 K vertices, F=256 backward 3.95 -> 4.07 ms;
        // 133 K vertices, F=128 1.16 -> 1.25), on the 2.45 M-vertex graph it does not (F=512 12.9 -> 11.6).
        if (bl.active && esz == 2 && bl.automatic && N < 8 * int64_t(32768)) bl.active = false;
        if (bl.active && edge_scale) {
            rc = gnn_plan_blocked_edge_scale(plan, src_mode, stream, &scale_blk);
            if (rc != GNN_OK) return rc;
        }
        if (bl.active && bound) {
            rc = gnn_plan_blocked_bound_weights(plan, stream, &w_blk);
            if (rc != GNN_OK) return rc;
        }
    }
    // Own-row term of the finalisation kernels: from the caller's matrix, or from the plan's layout when a
    // producer wrote the matrix there (then already multiplied by the factor the rows carry).
    const int fin_self_mode = (prepacked && factor_in_tables && orig_self_mode == kSelfInvPlus1) ? int(kSelfPlain) : orig_self_mode;
    auto own_row_src = [&](int64_t f0) {
        OwnRowSrc s{};
        if (orig) {
            s.G = static_cast<const char *>(orig) + f0 * esz;
            s.ldg = ldx;
        } else {
            s.tbl = tables;
            s.table_stride = layout.table_stride;
            s.main_cols = int32_t(F - layout.tail_elems);
            s.tail = tail_table;
            s.tail_ld = layout.tail_ld;
            s.rank = rank;
            s.col_off = int32_t(f0);
        }
        return s;
    };
    bool plain_hub_columns = false;   // some launch left its hub rows to hub_finalize_kernel
    int64_t plain_hub_col_begin = F;  // ... from this column on

    // The short rows of the blocked launches run on a second stream beside the pieces: they write other rows and
    // read the same tables, the pieces are bound by line requests that hit in the L2s and the short rows by the
    // misses behind them (2.45 M vertices: F=100 5.57 -> 5.32 ms, F=256 10.11 -> 9.98)
    hipStream_t side = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    if (bl.active && !(o.flags & GNN_FLAG_NO_SHORT_ROW_OVERLAP)) {
        side = overlap_stream();
        if (side && (hipEventCreateWithFlags(&fork, hipEventDisableTiming) != hipSuccess ||
                     hipEventCreateWithFlags(&join, hipEventDisableTiming) != hipSuccess)) {
            if (fork) (void)hipEventDestroy(fork);
            fork = join = nullptr;
            side = nullptr;
            (void)hipGetLastError();
        }
        if (side && (hipEventRecord(fork, stream) != hipSuccess || hipStreamWaitEvent(side, fork, 0) != hipSuccess)) {
            (void)hipEventDestroy(fork);
            (void)hipEventDestroy(join);
            return GNN_ERR_LAUNCH;
        }
    }
    auto finish_overlap = [&]() -> bool {  // the caller's stream waits for the second one; true = fine
        if (!side) return true;
        const bool ok = hipEventRecord(join, side) == hipSuccess && hipStreamWaitEvent(stream, join, 0) == hipSuccess;
        (void)hipEventDestroy(fork);  // released by the runtime once the recorded work has completed
        (void)hipEventDestroy(join);
        side = nullptr;
        return ok;
    };

    for (int gi = 0; gi < n_segs; ++gi) {
        const int64_t f0 = segs[gi].f0, fw = segs[gi].fw;
        const int log2_s = segs[gi].log2_s;
        const int64_t slice_cols = segs[gi].slice_cols;
        const int64_t strips = (slice_cols + vec - 1) / vec;
        const int log2_c = strips >= 64 ? 6 : gnn_ilog2_ceil(strips);
        const int C = 1 << log2_c;
        const int npass = int((strips + C - 1) / C);

        AggArgs a{};
        a.indptr = indptr;
        a.indices = gather_indices;
        a.w = w;
        // row-major: the segment starts f0 columns into every row; slice-major: at its first slice table
        a.X = static_cast<const char *>(gathered) + (slice_major ? (f0 / line_elems) * layout.table_stride : f0) * esz;
        a.slice_stride = slice_major ? layout.table_stride : 0;
        a.Y = static_cast<char *>(out) + f0 * esz;
        a.ldx = ldg;
        a.ldy = ldy;
        a.F = int32_t(fw);
        a.ip64 = o.indptr_is_64 ? 1 : 0;
        a.edge_scale = edge_scale;
        a.dst_mode = dst_mode;
        a.self_mode = self_mode;
        a.col_counts = plan ? plan->col_counts : nullptr;
        a.log2_slices = log2_s;
        a.slice_cols = int32_t(slice_cols);
        a.store_vec = store_vec;
        a.row_map = rank_indices ? rank : nullptr;
        a.p_indptr = rank_indices ? rl.p_indptr : nullptr;
        a.p_chunks = rank_indices ? rl.p_chunks : nullptr;
        a.cold_on = (o.flags & GNN_FLAG_NO_COLD_HINTS) ? 0 : 1;
        // Warm-set size, measured on the 2.45 M-vertex graph: with <= 4 slices per launch (two or more
        // XCDs share a slice) 8 x 32,768 rows is best (F=100: 5.81 ms against 6.03 at 5 x), with 8
        // slices 5-6 x (F=256: 12.18 ms against 12.28 at 8 x and 12.64 at 3 x).
        // Launches of one slice get none: no measurable effect on a whole line, and the dense tail loses
        // with it (8 rows share a line there: F=100 5.70 -> 5.88 ms).
        a.warm_rank = INT32_MAX;
        // With the long rows taken out as source-blocked pieces the hints stopped paying for the short rows that are
        // left (2.45 M vertices: F=100 5.32 -> 5.28 ms without them, F=256 the same either way, as with any warm set
        // from 12 x 32,768 rows up): they are kept for the launches that serve all rows.
        if (rank_indices && rl.cold_pays && log2_s > 0 && !bl.active) a.warm_rank = int32_t(32768) * (log2_s <= 2 ? 8 : 6);
        a.X_tail = tail_table;
        a.ld_tail = layout.tail_ld;
        a.tail_slice = segs[gi].tail_slice;
        a.bias = bias ? bias + f0 : nullptr;
        a.relu = relu;
        if (plan) {
            a.row_perm = plan->row_perm;
            a.chunks = plan->chunks;
            // The scratch rows are F wide for every slab; point at this slab's columns.
            a.partial = partial ? partial + f0 : nullptr;
            a.ldp = gnn_partial_ld(F);
        }
        const bool blocked = bl.active && segs[gi].tail_slice < 0;
        if (blocked) {
            const int line_floats = int(line_elems);
            int rc = gnn_plan_blocked_partial(plan, 1 << log2_s, line_floats);
            if (rc != GNN_OK) { finish_overlap(); return rc; }
            PieceArgs pa{};
            pa.pieces = bl.pieces;
            pa.n_pieces = bl.n_pieces;
            pa.idx = bl.indices;
            pa.epos = bl.epos;
            pa.idx16 = bl.idx16;
            pa.piece_block = bl.piece_block;
            pa.n_blocks = bl.n_blocks;
            pa.hot_lines = bl.hot_lines;
            pa.block_lines = bl.block_lines;
            pa.w = w;
            pa.w_blk = w_blk;
            pa.scale_blk = scale_blk;
            pa.X = a.X;
            pa.slice_stride = layout.table_stride;
            pa.partial = static_cast<float *>(plan->blk_partial);
            pa.log2_slices = log2_s;
            const int64_t pblocks = ((bl.n_pieces + 8 * kWavesPerBlock - 1) / (8 * kWavesPerBlock)) << log2_s;
            if (pblocks > INT32_MAX) { finish_overlap(); return GNN_ERR_UNSUPPORTED; }
            const int n_sl = 1 << log2_s;
            const dim3 pgrid(static_cast<unsigned>(pblocks)), fgrid(static_cast<unsigned>((bl.n_hot * n_sl * 8 + 255) / 256));
            const int32_t *hot_rows = plan->row_perm + bl.hot_begin;
            const OwnRowSrc own = own_row_src(f0);
            if (o.dtype == GNN_F32) {
                if (coef) piece_kernel<float, true><<<pgrid, kBlockThreads, 0, stream>>>(pa);
                else piece_kernel<float, false><<<pgrid, kBlockThreads, 0, stream>>>(pa);
                blk_finalize_kernel<float><<<fgrid, 256, 0, stream>>>(
                    hot_rows, bl.n_hot, bl.rowbase, pa.partial, bl.n_pieces, n_sl, indptr, o.indptr_is_64 ? 1 : 0, dst_mode,
                    static_cast<float *>(out) + f0, ldy, int(fw), store_vec, fin_self_mode, own,
                    plan->col_counts, bias ? bias + f0 : nullptr, relu);
            } else {
                if (coef) piece_kernel<bf16_t, true><<<pgrid, kBlockThreads, 0, stream>>>(pa);
                else piece_kernel<bf16_t, false><<<pgrid, kBlockThreads, 0, stream>>>(pa);
                blk_finalize_kernel<bf16_t><<<fgrid, 256, 0, stream>>>(
                    hot_rows, bl.n_hot, bl.rowbase, pa.partial, bl.n_pieces, n_sl, indptr, o.indptr_is_64 ? 1 : 0, dst_mode,
                    static_cast<bf16_t *>(out) + f0, ldy, int(fw), store_vec, fin_self_mode, own,
                    plan->col_counts, bias ? bias + f0 : nullptr, relu);
            }
            if (hipGetLastError() != hipSuccess) { finish_overlap(); return GNN_ERR_LAUNCH; }
        } else if (has_hub) {
            plain_hub_columns = true;
            if (f0 < plain_hub_col_begin) plain_hub_col_begin = f0;
        }
        int32_t nb = 0;
        int64_t next_block = gnn_fill_bins(a.bins, &nb, plan, N, log2_c, blocked ? bl.first_bin : INT32_MAX);
        a.n_bins = nb;
        if (nb == 0 || next_block == 0) continue;
        next_block <<= log2_s;
        if (next_block > INT32_MAX) { finish_overlap(); return GNN_ERR_UNSUPPORTED; }

        dim3 grid(static_cast<unsigned>(next_block));
        hipError_t err = hipSuccess;
        hipStream_t rows_stream = (blocked && side) ? side : stream;  // the short rows of a blocked launch may overlap the pieces
        if (o.dtype == GNN_F32) {
            if (vec == 4) err = launch_coef<float, 4>(coef, npass, grid, rows_stream, a);
            else if (vec == 2) err = launch_coef<float, 2>(coef, npass, grid, rows_stream, a);
            else err = launch_coef<float, 1>(coef, npass, grid, rows_stream, a);
        } else {
            if (vec == 8) err = launch_coef<bf16_t, 8>(coef, npass, grid, rows_stream, a);
            else if (vec == 4) err = launch_coef<bf16_t, 4>(coef, npass, grid, rows_stream, a);
            else if (vec == 2) err = launch_coef<bf16_t, 2>(coef, npass, grid, rows_stream, a);
            else err = launch_coef<bf16_t, 1>(coef, npass, grid, rows_stream, a);
        }
        if (err != hipSuccess) { finish_overlap(); return GNN_ERR_LAUNCH; }
    }

    if (!finish_overlap()) return GNN_ERR_LAUNCH;
    if (has_hub && plain_hub_columns) {
        const int64_t hub_begin = plan->bin_offsets[plan->n_bins - 1];
        dim3 grid(static_cast<unsigned>(plan->n_hub_rows));
        if (o.dtype == GNN_F32)
            hub_finalize_kernel<float><<<grid, 256, 0, stream>>>(plan->row_perm + hub_begin, plan->n_hub_rows, plan->hub_chunk_offsets,
                                                                 partial, indptr, o.indptr_is_64 ? 1 : 0, dst_mode,
                                                                 static_cast<float *>(out), ldy, int(F), gnn_partial_ld(F), fin_self_mode,
                                                                 own_row_src(0), plan->col_counts, bias, relu, int(plain_hub_col_begin));
        else
            hub_finalize_kernel<bf16_t><<<grid, 256, 0, stream>>>(plan->row_perm + hub_begin, plan->n_hub_rows, plan->hub_chunk_offsets,
                                                                  partial, indptr, o.indptr_is_64 ? 1 : 0, dst_mode,
                                                                  static_cast<bf16_t *>(out), ldy, int(F), gnn_partial_ld(F), fin_self_mode,
                                                                  own_row_src(0), plan->col_counts, bias, relu, int(plain_hub_col_begin));
        if (hipGetLastError() != hipSuccess) return GNN_ERR_LAUNCH;
    }
    return GNN_OK;
}

}  // namespace

// Copy of an fp32 matrix into rows of another stride (the plan-owned padded matrix), with the
// widest chunks the source allows (used by ap.hip).
int gnn_pad_rows_f32(const float *src, int64_t ld_src, float *dst, int64_t ld_dst, int64_t N, int64_t F, hipStream_t stream) {
    const int64_t row_bytes = F * 4, src_ld_bytes = ld_src * 4, dst_ld_bytes = ld_dst * 4;
    const uintptr_t addr = reinterpret_cast<uintptr_t>(src);
    hipError_t err;
    if (row_bytes % 16 == 0 && src_ld_bytes % 16 == 0 && addr % 16 == 0)
        err = launch_pad<u32x4>(src, src_ld_bytes, dst, dst_ld_bytes, N, row_bytes, stream);
    else if (row_bytes % 8 == 0 && src_ld_bytes % 8 == 0 && addr % 8 == 0)
        err = launch_pad<u32x2>(src, src_ld_bytes, dst, dst_ld_bytes, N, row_bytes, stream);
    else
        err = launch_pad<uint32_t>(src, src_ld_bytes, dst, dst_ld_bytes, N, row_bytes, stream);
    return err == hipSuccess ? GNN_OK : GNN_ERR_LAUNCH;
}

int gnn_packed_target_for(gnn_plan *plan, const void *indptr, const int32_t *indices, int64_t N, int64_t F, int op, bool backward,
                          bool force, hipStream_t stream, gnn_packed_target *out) {
    *out = gnn_packed_target{};
    if (!plan || !indptr || N <= 0 || F <= 0 || plan->n_rows != N || plan->n_edges <= 0) return GNN_OK;
    int src_mode = kScaleNone;
    if (op == GNN_MEAN && backward) src_mode = kScaleInv;
    else if (op == GNN_GCN_SYM) src_mode = kScaleRsqrt;
    else if (op == GNN_SAGE_GCN && backward) src_mode = kScaleInvPlus1;
    const gnn_layout layout = gnn_choose_layout(plan, N, F, 4, F, true, force ? GNN_FLAG_FORCE_PADDED_COPY : 0, force ? 8 : 0,
                                                /*allow_tail=*/true, /*scaled_source=*/src_mode != kScaleNone,
                                                gnn_plan_blocks_expected(plan, 4));
    if (!(layout.padded_copy && layout.slice_major)) return GNN_OK;  // that call gathers rows where they lie
    const int64_t lines = (F + 31) / 32;
    if (lines < 2 || lines > 256) return GNN_OK;
    int rc = gnn_plan_padded(plan, layout.bytes);
    if (rc != GNN_OK) return rc;
    gnn_rank_layout rl{};
    rc = gnn_plan_rank_indices(plan, indptr, indices, false, stream, &rl);
    if (rc != GNN_OK) return rc;
    if (!rl.rank) return GNN_OK;
    out->active = true;
    out->base = static_cast<float *>(plan->padded);
    out->table_stride = layout.table_stride;
    out->main_cols = int32_t(F - layout.tail_elems);
    out->tail = layout.tail_elems > 0 ? out->base + layout.main_lines * layout.table_stride : nullptr;
    out->tail_ld = layout.tail_ld;
    out->rank = rl.rank;
    out->counts = plan->col_counts;
    out->scale_mode = src_mode;
    return GNN_OK;
}

int gnn_aggregate_prepacked(const void *indptr, const int32_t *indices, void *out, int64_t N, int64_t F, int op,
                            const gnn_opts *opts, bool backward, bool force, const float *bias, int relu) {
    gnn_opts o{};
    if (opts) o = *opts;
    if (force) {
        o.flags |= GNN_FLAG_FORCE_PADDED_COPY;
        o.max_slices = 8;
    }
    return run_aggregate(indptr, indices, nullptr, nullptr, out, N, F, op, &o, backward, bias, relu, /*no_alloc=*/false,
                         /*prepacked=*/true);
}

// Caller-owned packed copies: the layout every packed call uses is the forced one (slice tables in rank
// order whatever the size of the graph), so that the size depends on N, F and the element size only.
static void packed_opts(const gnn_opts *opts, gnn_opts &o) {
    o = gnn_opts{};
    if (opts) o = *opts;
    o.flags = (o.flags | GNN_FLAG_FORCE_PADDED_COPY | GNN_FLAG_NO_DENSE_TAIL) &
              ~(GNN_FLAG_NO_PADDED_COPY | GNN_FLAG_NO_RANK_ORDER | GNN_FLAG_NO_COLUMN_SLICES | GNN_FLAG_NO_SLICE_TABLES);
    o.max_slices = 8;
}

extern "C" GNN_API int64_t gnn_packed_bytes(int64_t N, int64_t F, int dtype) {
    if (N <= 0 || F <= 0 || (dtype != GNN_F32 && dtype != GNN_BF16)) return 0;
    const int64_t esz = dtype == GNN_BF16 ? 2 : 4, line_elems = 128 / esz;
    const int64_t lines = (F + line_elems - 1) / line_elems;
    if (lines < 2 || lines > 256) return 0;  // rows of one line are not laid out as slice tables
    return N * lines * 128;
}

extern "C" GNN_API int gnn_pack_rows(const void *indptr, const int32_t *indices, const void *X, void *packed,
                                     int64_t packed_bytes, int64_t N, int64_t F, int op, int backward, const gnn_opts *opts) {
    gnn_opts o;
    packed_opts(opts, o);
    if (!packed || !X) return (N == 0 || F == 0) ? GNN_OK : GNN_ERR_INVALID_ARG;
    // `packed` stands in for the output argument, which a pack-only call never writes
    return run_aggregate(indptr, indices, nullptr, X, packed, N, F, op, &o, backward != 0, nullptr, 0, /*no_alloc=*/false,
                         /*prepacked=*/false, packed, packed_bytes, /*pack_only=*/true);
}

extern "C" GNN_API int gnn_aggregate_packed(const void *indptr, const int32_t *indices, const float *edge_w, const void *packed,
                                            int64_t packed_bytes, void *Y, int64_t N, int64_t F, int op, int backward,
                                            const gnn_opts *opts) {
    gnn_opts o;
    packed_opts(opts, o);
    if (!packed) return (N == 0 || F == 0) ? GNN_OK : GNN_ERR_INVALID_ARG;
    return run_aggregate(indptr, indices, edge_w, nullptr, Y, N, F, op, &o, backward != 0, nullptr, 0, /*no_alloc=*/false,
                         /*prepacked=*/true, const_cast<void *>(packed), packed_bytes, /*pack_only=*/false);
}

// Forward aggregation with the epilogue of a fused layer (used by layer.hip).
int gnn_aggregate_fwd_epilogue(const void *indptr, const int32_t *indices, const void *X, void *Y, int64_t N, int64_t F,
                               int op, const gnn_opts *opts, const float *bias, int relu) {
    return run_aggregate(indptr, indices, nullptr, X, Y, N, F, op, opts, /*backward=*/false, bias, relu);
}

extern "C" GNN_API int gnn_aggregate_fwd(const void *indptr, const int32_t *indices, const float *edge_w, const void *X,
                                 void *Y, int64_t N, int64_t F, int op, const gnn_opts *opts) {
    return run_aggregate(indptr, indices, edge_w, X, Y, N, F, op, opts, /*backward=*/false);
}

extern "C" GNN_API int gnn_aggregate_fwd_noalloc(const void *indptr, const int32_t *indices, const float *edge_w,
                                                 const void *X, void *Y, int64_t N, int64_t F, int op, const gnn_opts *opts) {
    return run_aggregate(indptr, indices, edge_w, X, Y, N, F, op, opts, /*backward=*/false, nullptr, 0, /*no_alloc=*/true);
}

extern "C" GNN_API int gnn_aggregate_bwd(const void *indptr_t, const int32_t *indices_t, const float *edge_w_t,
                                 const void *dY, void *dX, int64_t N, int64_t F, int op, const gnn_opts *opts) {
    return run_aggregate(indptr_t, indices_t, edge_w_t, dY, dX, N, F, op, opts, /*backward=*/true);
}
