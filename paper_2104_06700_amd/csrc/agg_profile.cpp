// Stand-alone driver for rocprofv3 counter runs (the profiler's counter mode does not
// survive the Python process on this image): loads a graph dumped by
// `bench.py --dump-graph DIR`, builds the plans and runs the forward and backward
// aggregation through the C ABI a few times, preceded by a 1 GiB streaming copy whose
// counter readings calibrate FETCH_SIZE / WRITE_SIZE.
//
// usage: agg_profile DIR OP(0|1|2|3) REPS [option ...] F [F ...]
// options: "bf16" (features in bf16 from there on; default fp32), "weights" (an explicit fp32 weight
// per edge, all equal, from there on; the array is bound to both plans as a static one, as the bench does),
// "noslice" switches the XCD column slicing off for the widths that follow it; "flags=N" sets
// gnn_opts.flags (GNN_FLAG_* bits) for the widths that follow it; "block=D,H,B,P,R" (anywhere) sets
// the source-blocking parameters of both plans (min_degree, hot_lines, block_lines, max_piece,
// rest_min_count; 0 = default, D = -1 switches blocking off).
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "gnnagg.h"

#define CHECK(x)                                                                   \
    do {                                                                           \
        if ((x) != hipSuccess) { fprintf(stderr, "HIP error at %s:%d\n", __FILE__, __LINE__); return 2; } \
    } while (0)
#define GCHECK(x)                                                                  \
    do {                                                                           \
        int s_ = (x);                                                              \
        if (s_ != GNN_OK) { fprintf(stderr, "gnnagg: %s at %s:%d\n", gnn_status_string(s_), __FILE__, __LINE__); return 3; } \
    } while (0)

static void *load_to_device(const std::string &path, size_t bytes) {
    std::vector<char> host(bytes);
    FILE *f = fopen(path.c_str(), "rb");
    if (!f) { fprintf(stderr, "cannot open %s\n", path.c_str()); return nullptr; }
    size_t got = fread(host.data(), 1, bytes, f);
    fclose(f);
    if (got != bytes) { fprintf(stderr, "short read on %s\n", path.c_str()); return nullptr; }
    void *d = nullptr;
    if (hipMalloc(&d, bytes ? bytes : 16) != hipSuccess) return nullptr;
    if (hipMemcpy(d, host.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) return nullptr;
    return d;
}

int main(int argc, char **argv) {
    if (argc < 5) { fprintf(stderr, "usage: %s DIR OP REPS F [F ...]\n", argv[0]); return 1; }
    const std::string dir = argv[1];
    const int op = atoi(argv[2]);
    const int reps = atoi(argv[3]);
    long long N = 0, E = 0; int ip64 = 0;
    {
        FILE *f = fopen((dir + "/meta.txt").c_str(), "r");
        if (!f || fscanf(f, "%lld %lld %d", &N, &E, &ip64) != 3) { fprintf(stderr, "bad meta.txt\n"); return 1; }
        fclose(f);
    }
    const size_t ipb = ip64 ? 8 : 4;
    void *indptr = load_to_device(dir + "/indptr.bin", ipb * (N + 1));
    void *indices = load_to_device(dir + "/indices.bin", 4 * (size_t)E);
    void *indptr_t = load_to_device(dir + "/indptr_t.bin", ipb * (N + 1));
    void *indices_t = load_to_device(dir + "/indices_t.bin", 4 * (size_t)E);
    if (!indptr || !indices || !indptr_t || !indices_t) return 2;

    // calibration copy: 1 GiB read + 1 GiB write
    {
        void *a = nullptr, *b = nullptr;
        const size_t n = size_t(1) << 30;
        CHECK(hipMalloc(&a, n)); CHECK(hipMalloc(&b, n));
        CHECK(hipMemset(a, 0x3c, n));
        for (int i = 0; i < 3; ++i) GCHECK(gnn_calib_copy(a, b, (int64_t)n, nullptr));
        CHECK(hipDeviceSynchronize());
        CHECK(hipFree(a)); CHECK(hipFree(b));
    }

    gnn_plan *pf = nullptr, *pb = nullptr;
    GCHECK(gnn_plan_create(indptr, (const int32_t *)indices, N, ip64, nullptr, nullptr, &pf));
    GCHECK(gnn_plan_create(indptr_t, (const int32_t *)indices_t, N, ip64, nullptr, nullptr, &pb));
    for (int a = 4; a < argc; ++a) {
        if (std::string(argv[a]).rfind("block=", 0) != 0) continue;
        gnn_blocking_params bp{};
        long long v[5] = {0, 0, 0, 0, 0};
        sscanf(argv[a] + 6, "%lld,%lld,%lld,%lld,%lld", &v[0], &v[1], &v[2], &v[3], &v[4]);
        bp.min_degree = v[0]; bp.hot_lines = v[1]; bp.block_lines = v[2]; bp.max_piece = v[3]; bp.rest_min_count = v[4];
        GCHECK(gnn_plan_set_blocking(pf, &bp));
        GCHECK(gnn_plan_set_blocking(pb, &bp));
    }

    int flags = 0, max_slices = 0, esz = 4;
    float *w = nullptr;
    for (int a = 4; a < argc; ++a) {
        if (std::string(argv[a]) == "bf16") { esz = 2; continue; }
        if (std::string(argv[a]) == "weights") {
            if (!w) {
                CHECK(hipMalloc(&w, 4 * (size_t)E));
                CHECK(hipMemset(w, 0x3c, 4 * (size_t)E));
                GCHECK(gnn_plan_bind_edge_weights(pf, w, nullptr));
                GCHECK(gnn_plan_bind_edge_weights(pb, w, nullptr));
            }
            continue;
        }
        if (std::string(argv[a]) == "noslice") { flags = GNN_FLAG_NO_COLUMN_SLICES; continue; }
        if (std::string(argv[a]).rfind("flags=", 0) == 0) { flags = atoi(argv[a] + 6); continue; }
        if (std::string(argv[a]).rfind("slices=", 0) == 0) { max_slices = atoi(argv[a] + 7); continue; }
        if (std::string(argv[a]).rfind("block=", 0) == 0) continue;
        const long long F = atoll(argv[a]);
        const size_t bytes = (size_t)N * F * esz;
        void *X = nullptr, *Y = nullptr;
        CHECK(hipMalloc(&X, bytes)); CHECK(hipMalloc(&Y, bytes));
        CHECK(hipMemset(X, 0x3c, bytes));
        gnn_opts o{};
        o.indptr_is_64 = ip64;
        o.dtype = esz == 2 ? GNN_BF16 : GNN_F32;
        o.flags = flags;
        o.max_slices = max_slices;
        o.plan = pf;
        hipEvent_t e0, e1;
        CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
        GCHECK(gnn_aggregate_fwd(indptr, (const int32_t *)indices, w, X, Y, N, F, op, &o));  // warm-up
        CHECK(hipEventRecord(e0, nullptr));
        for (int r = 0; r < reps; ++r) GCHECK(gnn_aggregate_fwd(indptr, (const int32_t *)indices, w, X, Y, N, F, op, &o));
        CHECK(hipEventRecord(e1, nullptr));
        CHECK(hipEventSynchronize(e1));
        float ms_f = 0; CHECK(hipEventElapsedTime(&ms_f, e0, e1));
        o.plan = pb;
        GCHECK(gnn_aggregate_bwd(indptr_t, (const int32_t *)indices_t, w, X, Y, N, F, op, &o));
        CHECK(hipEventRecord(e0, nullptr));
        for (int r = 0; r < reps; ++r) GCHECK(gnn_aggregate_bwd(indptr_t, (const int32_t *)indices_t, w, X, Y, N, F, op, &o));
        CHECK(hipEventRecord(e1, nullptr));
        CHECK(hipEventSynchronize(e1));
        float ms_b = 0; CHECK(hipEventElapsedTime(&ms_b, e0, e1));
        printf("N=%lld E=%lld F=%lld %s%s op=%d flags=%d slices<=%d calls=%d fwd %.4f ms  bwd %.4f ms  (%.1f / %.1f GEF/s)\n", N, E, F, esz == 2 ? "bf16" : "fp32", w ? " weighted" : "", op, flags, max_slices, 2 * (reps + 1), ms_f / reps,
               ms_b / reps, E * F / (ms_f / reps) / 1e6, E * F / (ms_b / reps) / 1e6);
        CHECK(hipFree(X)); CHECK(hipFree(Y));
    }
    {
        int64_t r = 0, e = 0, pc = 0; int32_t nb = 0;
        gnn_plan_blocked_sizes(pf, &r, &e, &pc, &nb);
        printf("source blocks (forward plan): %lld rows, %lld edges, %lld pieces, %d blocks\n", (long long)r, (long long)e, (long long)pc, nb);
    }
    gnn_plan_destroy(pf);
    gnn_plan_destroy(pb);
    return 0;
}
