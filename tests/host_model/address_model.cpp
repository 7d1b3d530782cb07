// Address model of the library: the product sources compiled for the host (see stub/hip/hip_runtime.h) and
// driven through the C ABI with heap buffers of exactly the sizes a caller would allocate, under
// AddressSanitizer and UBSan.  Any global-memory access outside its tensor aborts the run with a report
// that names the access; "transfers" (global -> LDS) are range-checked the way the buffer descriptor does it.
//
//   address_model random <seed> <cases>     layers of random shape in every alignment class, 1-4 per case, gate
//                                           vectors sliced at arbitrary offsets out of one array: plain calls, then
//                                           flop_fwd_sampling / flop_bwd_deferred / flop_bwd_boundary, then the
//                                           indexed active-rank calls (gathered rows, scattered output rows)
//   address_model classes [stride]          a fixed sweep (every stride-th case of it): every combination of alignment class of d, r, dout
//                                           (odd, 2 mod 4, 4 mod 8, 0 mod 8) with dense last rows, riders on
//                                           and off, empty pending lists, boundary jobs with and without new gates
//
//   address_model padded                    rows padded to 16 bytes around extents that are not multiples of 8 elements
//   address_model lowrank                   flop_fwd on layers whose second product takes the kernel for ranks up to 256
//
//   address_model case <bf16|f32> <extra> n d r dout [n d r dout ...]   the given layers, with and without new gates, every block shape
//
// Prints one line per case before running it, so that a report names its case.
#include "../../paper_1910_04732_amd/csrc/flop_api.hip"
#include "../../paper_1910_04732_amd/csrc/flop_bench.hip"

#include <random>
#include <string>

namespace {

struct Rng {
    std::mt19937_64 g;
    explicit Rng(uint64_t s) : g(s) {}
    int64_t range(int64_t lo, int64_t hi) { return lo + (int64_t)(g() % (uint64_t)(hi - lo)); }   // [lo, hi)
    template <typename T, size_t N> T pick(const T (&a)[N]) { return a[g() % N]; }
    double uni() { return (double)(g() >> 11) / 9007199254740992.0; }
};

// A "device" allocation as torch's allocator hands it out: 512-byte aligned, here of exactly the bytes asked
// for, so that the sanitizer's red zone starts at the tensor's last byte.
struct Buf {
    void* p = nullptr;
    size_t bytes = 0;
    Buf() = default;
    explicit Buf(size_t n, int fill = 0) : bytes(n)
    {
        if (posix_memalign(&p, 512, n ? n : 1) != 0) abort();
        memset(p, fill, n);
    }
    Buf(const Buf&) = delete;
    Buf& operator=(const Buf&) = delete;
    Buf(Buf&& o) noexcept : p(o.p), bytes(o.bytes) { o.p = nullptr; }
    Buf& operator=(Buf&& o) noexcept { free(p); p = o.p; bytes = o.bytes; o.p = nullptr; return *this; }
    ~Buf() { free(p); }
    float* f() const { return (float*)p; }
};

Buf gates(int64_t n, float v)
{
    Buf b((size_t)n * 4);
    for (int64_t i = 0; i < n; ++i) b.f()[i] = v;
    return b;
}

int must(int rc, const char* what)
{
    if (rc != FLOP_OK) { fprintf(stderr, "%s returned %d (%s)\n", what, rc, flop_status_string(rc)); abort(); }
    return rc;
}

struct Layer {
    int64_t n, d, r, dout, off;
    Buf x, Q, P, dy, g, y, dx, dQ, dP, da, ws;
};

Layer make_layer(flop_dtype dt, int64_t n, int64_t d, int64_t r, int64_t dout, int64_t off)
{
    const size_t es = dt == FLOP_BF16 ? 2 : 4;
    Layer L;
    L.n = n; L.d = d; L.r = r; L.dout = dout; L.off = off;
    L.x = Buf(n * d * es); L.Q = Buf(r * d * es); L.P = Buf(dout * r * es); L.dy = Buf(n * dout * es);
    L.g = Buf(n * r * es); L.y = Buf(n * dout * es);
    L.dx = Buf(n * d * es); L.dQ = Buf(r * d * es); L.dP = Buf(dout * r * es); L.da = Buf(r * 4);
    L.ws = Buf(flop_workspace_bytes(FLOP_OP_BWD, dt, n, d, r, dout));
    return L;
}

const flop_hc kHc = {2.0f / 3.0f, -0.1f, 1.1f};

// Dense row-major tensors: leading dimension = row length.
void plain_pass(flop_dtype dt, std::vector<Layer>& layers, int64_t G, const float* la, const float* u, const float* w)
{
    Buf z = gates(G, 0.5f), dz = gates(G, 0.1f), l0(4), l0g((size_t)G * 4);
    Buf gws(flop_workspace_bytes(FLOP_OP_EXPECTED_L0, FLOP_F32, G, 0, 0, 0));
    must(flop_gate_sample_l0(la, u, G, kHc, z.f(), dz.f(), w, l0.f(), l0g.f(), gws.p, gws.bytes, nullptr), "flop_gate_sample_l0");
    for (Layer& t : layers) {
        must(flop_fwd(dt, t.n, t.d, t.r, t.dout, t.x.p, t.d, t.Q.p, t.d, t.P.p, t.r, z.f() + t.off, t.g.p, t.r, t.y.p, t.dout,
                      nullptr, 0, nullptr), "flop_fwd");
        must(flop_bwd(dt, t.n, t.d, t.r, t.dout, t.dy.p, t.dout, t.x.p, t.d, t.Q.p, t.d, t.P.p, t.r, z.f() + t.off,
                      dz.f() + t.off, t.g.p, t.r, t.dx.p, t.d, t.dQ.p, t.d, t.dP.p, t.r, t.da.f(), 0, t.ws.p, t.ws.bytes, nullptr),
             "flop_bwd");
        if (flop_workspace_bytes(FLOP_OP_BWD, dt, t.n, t.d, t.r, t.dout) <= FLOP_STATIC_SCRATCH_BYTES)
            must(flop_bwd_static(dt, t.n, t.d, t.r, t.dout, t.dy.p, t.dout, t.x.p, t.d, t.Q.p, t.d, t.P.p, t.r, z.f() + t.off,
                                 dz.f() + t.off, t.g.p, t.r, t.dx.p, t.d, t.dQ.p, t.d, t.dP.p, t.r, t.da.f(), 0, nullptr),
                 "flop_bwd_static");
    }
}

// The riding entry points in the order of a training step: sampling rides on the first layer's forward, the
// earlier layers' gate gradients are deferred, the boundary rides on the first layer's backward.
// next_gates: the boundary also samples the following step's gates (into buffers of their own).
void riding_pass(flop_dtype dt, std::vector<Layer>& layers, int64_t G, const float* la, const float* u, const float* w,
                 bool next_gates)
{
    Buf z = gates(G, 0.5f), dz = gates(G, 0.1f), l0(4), l0g((size_t)G * 4);
    Buf z2 = gates(G, 0.5f), dz2 = gates(G, 0.1f), l02(4), l0g2((size_t)G * 4);
    Buf gws(flop_workspace_bytes(FLOP_OP_EXPECTED_L0, FLOP_F32, G, 0, 0, 0));
    for (size_t i = 0; i < layers.size(); ++i) {
        Layer& t = layers[i];
        if (i == 0) {
            const flop_boundary_job job = {nullptr, 0, la, u, G, kHc, z.f(), dz.f(), w, l0.f(), l0g.f(), gws.p, gws.bytes};
            must(flop_fwd_sampling(dt, t.n, t.d, t.r, t.dout, t.x.p, t.d, t.Q.p, t.d, t.P.p, t.r, &job, t.off, t.g.p, t.r,
                                   t.y.p, t.dout, nullptr, 0, nullptr), "flop_fwd_sampling");
        } else {
            must(flop_fwd(dt, t.n, t.d, t.r, t.dout, t.x.p, t.d, t.Q.p, t.d, t.P.p, t.r, z.f() + t.off, t.g.p, t.r, t.y.p,
                          t.dout, nullptr, 0, nullptr), "flop_fwd");
        }
    }
    std::vector<flop_gate_grad_pending> pend;
    for (size_t i = layers.size(); i-- > 0;) {
        Layer& t = layers[i];
        if (i > 0) {
            flop_gate_grad_pending p;
            must(flop_bwd_deferred(dt, t.n, t.d, t.r, t.dout, t.dy.p, t.dout, t.x.p, t.d, t.Q.p, t.d, t.P.p, t.r, z.f() + t.off,
                                   dz.f() + t.off, t.g.p, t.r, t.dx.p, t.d, t.dQ.p, t.d, t.dP.p, t.r, t.da.f(), 0, t.ws.p,
                                   t.ws.bytes, nullptr, &p), "flop_bwd_deferred");
            pend.push_back(p);
        } else {
            flop_boundary_job job = {pend.data(), (int32_t)pend.size(), nullptr, nullptr, 0, kHc, nullptr, nullptr, nullptr,
                                     nullptr, nullptr, nullptr, 0};
            if (next_gates)
                job = {pend.data(), (int32_t)pend.size(), la, u, G, kHc, z2.f(), dz2.f(), w, l02.f(), l0g2.f(), gws.p, gws.bytes};
            must(flop_bwd_boundary(dt, t.n, t.d, t.r, t.dout, t.dy.p, t.dout, t.x.p, t.d, t.Q.p, t.d, t.P.p, t.r, z.f() + t.off,
                                   dz.f() + t.off, t.g.p, t.r, t.dx.p, t.d, t.dQ.p, t.d, t.dP.p, t.r, t.da.f(), 0, t.ws.p,
                                   t.ws.bytes, &job, nullptr), "flop_bwd_boundary");
        }
    }
}

// The open components read in place (flop_fwd_active_indexed / flop_bwd_active_indexed): every third component
// closed, the index list written here (the scan kernel's values are not modelled), P held transposed.  Rows of
// Q and Pt gathered by the list, output rows of dQ and dPt scattered by it, closed rows zeroed.
void indexed_pass(flop_dtype dt, std::vector<Layer>& layers)
{
    const size_t es = dt == FLOP_BF16 ? 2 : 4;
    for (Layer& t : layers) {
        Buf idx((size_t)t.r * 4), r_act(4), zc = gates(t.r, 0.5f), dzc = gates(t.r, 0.1f);
        int32_t cnt = 0;
        for (int64_t k = 0; k < t.r; ++k)
            if (k % 3 != 1) ((int32_t*)idx.p)[cnt++] = (int32_t)k;
        *(int32_t*)r_act.p = cnt;
        Buf Pt((size_t)t.r * t.dout * es), dPt((size_t)t.r * t.dout * es);
        must(flop_fwd_active_indexed(dt, t.n, t.d, t.r, t.dout, t.x.p, t.d, t.Q.p, t.d, Pt.p, t.dout, zc.f(),
                                     (const int32_t*)idx.p, (const int32_t*)r_act.p, t.g.p, t.r, t.y.p, t.dout, nullptr),
             "flop_fwd_active_indexed");
        must(flop_bwd_active_indexed(dt, t.n, t.d, t.r, t.dout, t.dy.p, t.dout, t.x.p, t.d, t.Q.p, t.d, Pt.p, t.dout, zc.f(),
                                     dzc.f(), (const int32_t*)idx.p, (const int32_t*)r_act.p, t.g.p, t.r, t.dx.p, t.d,
                                     t.dQ.p, t.d, dPt.p, t.dout, t.da.f(), 0, t.ws.p, t.ws.bytes, nullptr),
             "flop_bwd_active_indexed");
    }
}

// Weight gradients left out of every layer's backward call and computed afterwards in shared launches
// (flop_bwd_defer_weights / flop_weight_grad_finish): up to eight products of different layers in one grid.
void deferred_weights_pass(flop_dtype dt, std::vector<Layer>& layers)
{
    std::vector<flop_gate_grad_pending> gate_items(layers.size());
    std::vector<flop_weight_grad_pending> weight_items(layers.size());
    for (size_t i = 0; i < layers.size(); ++i) {
        Layer& t = layers[i];
        Buf z = gates(t.r, 0.5f), dz = gates(t.r, 0.1f);
        must(flop_bwd_defer_weights(dt, t.n, t.d, t.r, t.dout, t.dy.p, t.dout, t.x.p, t.d, t.Q.p, t.d, t.P.p, t.r, z.f(), dz.f(),
                                    t.g.p, t.r, t.dx.p, t.d, i % 3 == 2 ? nullptr : t.dQ.p, t.d, t.dP.p, t.r, t.da.f(), 0,
                                    t.ws.p, t.ws.bytes, nullptr, &gate_items[i], &weight_items[i]), "flop_bwd_defer_weights");
    }
    // the same list twice over, so that a single layer also meets launches shared with copies of itself
    std::vector<flop_weight_grad_pending> twice(weight_items);
    twice.insert(twice.end(), weight_items.begin(), weight_items.end());
    must(flop_weight_grad_finish(twice.data(), (int32_t)twice.size(), nullptr), "flop_weight_grad_finish");
    must(flop_weight_grad_finish(weight_items.data(), 1, nullptr), "flop_weight_grad_finish (one layer)");
}

void run_case(flop_dtype dt, const std::vector<std::array<int64_t, 4>>& shapes, int64_t extra, bool next_gates)
{
    std::vector<Layer> layers;
    int64_t off = 0;
    for (const auto& s : shapes) { layers.push_back(make_layer(dt, s[0], s[1], s[2], s[3], off)); off += s[2]; }
    const int64_t G = off + extra;
    Buf la = gates(G, 0.3f), u = gates(G, 0.4f), w = gates(G, 2.0f);
    plain_pass(dt, layers, G, la.f(), u.f(), w.f());
    riding_pass(dt, layers, G, la.f(), u.f(), w.f(), next_gates);
    indexed_pass(dt, layers);
    deferred_weights_pass(dt, layers);
}

std::string describe(flop_dtype dt, const std::vector<std::array<int64_t, 4>>& shapes, int64_t extra, bool next_gates)
{
    std::string s = dt == FLOP_BF16 ? "bf16" : "f32";
    for (const auto& q : shapes)
        s += " (" + std::to_string(q[0]) + "," + std::to_string(q[1]) + "," + std::to_string(q[2]) + "," + std::to_string(q[3]) + ")";
    s += " extra " + std::to_string(extra) + (next_gates ? " next-gates" : "");
    return s;
}

int run_random(uint64_t seed, int cases)
{
    Rng rng(seed);
    for (int c = 0; c < cases; ++c) {
        const int L = (int)rng.range(1, 5);
        const flop_dtype dt = rng.uni() < 0.8 ? FLOP_BF16 : FLOP_F32;
        std::vector<std::array<int64_t, 4>> shapes;
        for (int i = 0; i < L; ++i) {
            const int64_t n = rng.range(1, 1500);
            int64_t v[3] = {rng.range(1, 700), rng.range(1, 700), rng.range(1, 700)};
            static const int64_t aligns[4] = {1, 2, 8, 64};
            const int64_t a = rng.pick(aligns);
            for (int64_t& q : v) q += (a - q % a) % a;
            shapes.push_back({n, v[0], v[1], v[2]});
        }
        static const int64_t extras[4] = {0, 0, 3000, 5000};
        const int64_t extra = rng.pick(extras);
        const bool next_gates = rng.uni() < 0.3;
        const int shape = (int)rng.range(-1, flop_bench_tile_shapes());   // block shape of the bf16 transfer kernel
        must(flop_bench_force_tile_shape(shape), "flop_bench_force_tile_shape");
        printf("case %d %s shape %s\n", c, describe(dt, shapes, extra, next_gates).c_str(), flop_bench_tile_shape_name(shape));
        fflush(stdout);
        run_case(dt, shapes, extra, next_gates);
    }
    return 0;
}

// every stride-th case of the sweep (1 = all 1728)
int run_classes(int stride)
{
    // row lengths of every alignment class around one and two tiles, dense rows (a dense last row ends its tensor)
    static const int64_t dims[] = {1, 7, 30, 66, 68, 72, 129, 130, 132, 136, 200, 258};
    static const int64_t ns[] = {1, 63, 64, 65, 130, 257};
    int c = 0;
    for (int64_t d : dims)
        for (int64_t r : dims)
            for (int64_t dout : dims) {
                if (c % stride) { ++c; continue; }
                const int64_t n = ns[c % 6];
                const std::vector<std::array<int64_t, 4>> one = {{n, d, r, dout}};
                const std::vector<std::array<int64_t, 4>> two = {{n, d, r, dout}, {ns[(c + 1) % 6], dout, r, d}};
                const int shape = (c / stride) % (flop_bench_tile_shapes() + 1) - 1;
                must(flop_bench_force_tile_shape(shape), "flop_bench_force_tile_shape");
                printf("class %d %s shape %s\n", c, describe(FLOP_BF16, c % 3 ? one : two, c % 5 ? 0 : 37, c % 2).c_str(),
                       flop_bench_tile_shape_name(shape));
                fflush(stdout);
                run_case(FLOP_BF16, c % 3 ? one : two, c % 5 ? 0 : 37, c % 2);
                ++c;
            }
    return 0;
}

// The store-bound kernel for ranks up to 256 (y = g P^T with a short contraction): outputs large enough for the
// library to choose it, rows padded to 16 bytes, ranks that end inside a 16-byte piece, ragged row and column
// tails.  Every tensor ends where the interface allows it to: at the next multiple of 16 bytes after its last row's
// last element (include/flop.h: every row, the last included, is addressable that far).
int run_lowrank()
{
    static const int64_t cases[][4] = {   // n, d, r, dout
        {4100, 72, 64, 2050}, {4099, 40, 41, 2051}, {8200, 40, 100, 8200}, {8195, 24, 200, 8201}, {8200, 24, 250, 8190},
    };
    const size_t es = 2;
    for (const auto& c : cases) {
        const int64_t n = c[0], d = c[1], r = c[2], dout = c[3];
        auto ld = [](int64_t cols) { return (cols + 7) / 8 * 8; };
        auto bytes = [&](int64_t rows, int64_t cols) { return (size_t)((rows - 1) * ld(cols) + (cols + 7) / 8 * 8) * es; };
        printf("lowrank n=%ld d=%ld r=%ld dout=%ld\n", (long)n, (long)d, (long)r, (long)dout);
        fflush(stdout);
        Buf x(bytes(n, d)), Q(bytes(r, d)), P(bytes(dout, r)), g(bytes(n, r)), y(bytes(n, dout)), z = gates(r, 0.5f);
        const unsigned long before = flop_model::g_launch.launches;
        must(flop_fwd(FLOP_BF16, n, d, r, dout, x.p, ld(d), Q.p, ld(d), P.p, ld(r), z.f(), g.p, ld(r), y.p, ld(dout), nullptr, 0,
                      nullptr), "flop_fwd");
        if (flop_model::g_launch.launches != before + 2) { fprintf(stderr, "expected two launches\n"); return 1; }
    }
    return 0;
}

// Rows padded to 16 bytes around extents that are not multiples of 8 elements (the 410-wide matrices of a
// Transformer layer in rows of 416, compacted ranks inside a wider buffer): the 16-byte transfer kernels read whole
// chunks, so a row's last chunk reaches into its padding.  Tensors end at the next multiple of 16 bytes after the
// last row's last element, as the interface allows.  Forward, backward and the deferred weight gradients, every
// block shape.
int run_padded()
{
    static const int64_t cases[][5] = {   // n, d, r, dout, extra elements of padding per row (multiple of 8)
        {300, 203, 131, 77, 0}, {129, 410, 410, 1230, 0}, {257, 61, 306, 135, 8}, {70, 9, 3, 5, 0}, {333, 1029, 45, 67, 16},
    };
    const size_t es = 2;
    for (const auto& c : cases)
        for (int shape = -1; shape < flop_bench_tile_shapes(); ++shape) {
            const int64_t n = c[0], d = c[1], r = c[2], dout = c[3], pad = c[4];
            auto ld = [&](int64_t cols) { return (cols + 7) / 8 * 8 + pad; };
            auto mk = [&](int64_t rows, int64_t cols) { return Buf((size_t)((rows - 1) * ld(cols) + (cols + 7) / 8 * 8) * es); };
            must(flop_bench_force_tile_shape(shape), "flop_bench_force_tile_shape");
            printf("padded n=%ld d=%ld r=%ld dout=%ld pad=%ld shape %s\n", (long)n, (long)d, (long)r, (long)dout, (long)pad,
                   flop_bench_tile_shape_name(shape));
            fflush(stdout);
            Buf x = mk(n, d), Q = mk(r, d), P = mk(dout, r), dy = mk(n, dout), g = mk(n, r), y = mk(n, dout), dx = mk(n, d),
                dQ = mk(r, d), dP = mk(dout, r), da((size_t)r * 4), z = gates(r, 0.5f), dz = gates(r, 0.1f);
            Buf ws(flop_workspace_bytes(FLOP_OP_BWD, FLOP_BF16, n, d, r, dout));
            must(flop_fwd(FLOP_BF16, n, d, r, dout, x.p, ld(d), Q.p, ld(d), P.p, ld(r), z.f(), g.p, ld(r), y.p, ld(dout), nullptr, 0,
                          nullptr), "flop_fwd");
            must(flop_bwd(FLOP_BF16, n, d, r, dout, dy.p, ld(dout), x.p, ld(d), Q.p, ld(d), P.p, ld(r), z.f(), dz.f(), g.p, ld(r),
                          dx.p, ld(d), dQ.p, ld(d), dP.p, ld(r), da.f(), 0, ws.p, ws.bytes, nullptr), "flop_bwd");
            flop_gate_grad_pending gi;
            flop_weight_grad_pending wi;
            must(flop_bwd_defer_weights(FLOP_BF16, n, d, r, dout, dy.p, ld(dout), x.p, ld(d), Q.p, ld(d), P.p, ld(r), z.f(), dz.f(),
                                        g.p, ld(r), dx.p, ld(d), dQ.p, ld(d), dP.p, ld(r), da.f(), 0, ws.p, ws.bytes, nullptr, &gi,
                                        &wi), "flop_bwd_defer_weights");
            must(flop_weight_grad_finish(&wi, 1, nullptr), "flop_weight_grad_finish");
            const flop_gate_grad_pending items[1] = {gi};
            must(flop_gate_grad_finish(items, 1, nullptr), "flop_gate_grad_finish");
        }
    must(flop_bench_force_tile_shape(-1), "flop_bench_force_tile_shape");
    return 0;
}

}  // namespace

int main(int argc, char** argv)
{
    int rc = 2;
    if (argc >= 4 && !strcmp(argv[1], "random")) rc = run_random(strtoull(argv[2], nullptr, 10), atoi(argv[3]));
    else if (argc >= 2 && !strcmp(argv[1], "lowrank")) rc = run_lowrank();
    else if (argc >= 2 && !strcmp(argv[1], "padded")) rc = run_padded();
    else if (argc >= 2 && !strcmp(argv[1], "classes")) rc = run_classes(argc >= 3 ? std::max(1, atoi(argv[2])) : 1);
    else if (argc >= 8 && !strcmp(argv[1], "case") && (argc - 4) % 4 == 0) {   // case <bf16|f32> <extra gates> n d r dout ...
        std::vector<std::array<int64_t, 4>> shapes;
        for (int i = 4; i + 3 < argc; i += 4) shapes.push_back({atoll(argv[i]), atoll(argv[i + 1]), atoll(argv[i + 2]), atoll(argv[i + 3])});
        const flop_dtype dt = !strcmp(argv[2], "f32") ? FLOP_F32 : FLOP_BF16;
        for (int shape = -1; shape < flop_bench_tile_shapes(); ++shape)
            for (int next = 0; next < 2; ++next) {
                must(flop_bench_force_tile_shape(shape), "flop_bench_force_tile_shape");
                printf("case %s shape %s\n", describe(dt, shapes, atoll(argv[3]), next != 0).c_str(), flop_bench_tile_shape_name(shape));
                fflush(stdout);
                run_case(dt, shapes, atoll(argv[3]), next != 0);
            }
        rc = 0;
    }
    else fprintf(stderr, "usage: address_model random <seed> <cases> | classes [stride] | lowrank | padded | case <bf16|f32> <extra gates> n d r dout ...\n");
    if (rc == 0)
        printf("address model ok: %lu launches, %lu blocks, %lu transfers (%lu zero-filled)\n", flop_model::g_launch.launches,
               flop_model::g_launch.blocks, flop_model::g_launch.transfers, flop_model::g_launch.transfers_zero_filled);
    return rc;
}
