// TEST INFRASTRUCTURE ONLY: drives the host side of libaiq (built for the CPU against hip_stub.cpp) and the
// oracle (oracle.c) through their C entry points under AddressSanitizer + UndefinedBehaviorSanitizer.
// Input: a file of layer graphs written by the test (int32 count; per graph int32 n_layers and
// n_layers x 13 int32 descriptor fields).  Exit status 0 = every call returned what was expected; any
// sanitizer report aborts the run.
#include "../../include/aiq.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <random>
#include <memory>
#include <vector>

extern "C" {
long aiq_stub_launch_count();
int oracle_quantize_weights(const float *, int, int, int, float *, float *, int32_t *);
int oracle_quantize_weights_per_tensor(const float *, int, int, int, float *, float *, int32_t *);
int oracle_layer_ai(const int32_t *, int, const uint8_t *, int, int, double *, double *, double *);
int oracle_check_graph(const int32_t *, int, int, int, int);
int oracle_forward(const int32_t *, int, const float *const *, const float *const *, const float *, int, double *,
                   int32_t *, double *, int64_t *);
int oracle_eval_schemes_ex(const int32_t *, int, const float *const *, const float *const *, const float *, int,
                           const uint8_t *, int, int, int, double *, int32_t *, double *, int32_t *, int32_t *);
}

static int g_fail = 0;
#define EXPECT(cond)                                                         \
    do {                                                                     \
        if (!(cond)) {                                                       \
            std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond);    \
            ++g_fail;                                                        \
        }                                                                    \
    } while (0)

struct Buf { // exact-size, 256-byte aligned: the sanitizer's red zone starts at the first byte past it
    void *p = nullptr;
    size_t n = 0;
    explicit Buf(size_t bytes) : n(bytes)
    {
        const size_t rounded = (bytes + 255) / 256 * 256;
        p = std::aligned_alloc(256, rounded ? rounded : 256);
    }
    ~Buf() { std::free(p); }
    Buf(const Buf &) = delete;
};

static const uint8_t kBits[6] = {32, 16, 8, 6, 4, 2};

struct Graph {
    std::vector<aiq_layer_desc> d;
    std::vector<std::vector<float>> w, b;
    std::vector<const float *> wp, bp;
    int L = 0, classes = 0;
    size_t img_elems = 0;
};

static Graph make_graph(const int32_t *fields, int n, std::mt19937 &rng)
{
    Graph g;
    std::uniform_real_distribution<float> u(-1.f, 1.f);
    g.d.resize(n);
    std::memcpy(g.d.data(), fields, sizeof(aiq_layer_desc) * n);
    for (int l = 0; l < n; ++l) {
        const aiq_layer_desc &d = g.d[l];
        const size_t k = d.kind == 2 ? d.cin : (size_t)(d.kind == 1 ? 1 : d.cin) * d.kh * d.kw;
        g.w.emplace_back((size_t)d.cout * k);
        g.b.emplace_back((size_t)d.cout);
        for (float &v : g.w.back()) v = u(rng) * 0.1f;
        for (float &v : g.b.back()) v = u(rng) * 0.1f;
        g.L = std::max(g.L, d.scheme_slot + 1);
    }
    for (int l = 0; l < n; ++l) {
        g.wp.push_back(g.w[l].data());
        g.bp.push_back(g.b[l].data());
    }
    g.classes = g.d[n - 1].cout;
    g.img_elems = (size_t)g.d[0].hin * g.d[0].win * g.d[0].cin;
    return g;
}

static void run_library(const Graph &g, uint32_t flags, std::mt19937 &rng)
{
    const int n_layers = (int)g.d.size(), L = g.L;
    aiq_model *m = nullptr;
    aiq_status st = aiq_model_create_ex(g.d.data(), n_layers, g.wp.data(), g.bp.data(), flags, &m);
    EXPECT(st == AIQ_OK && m);
    if (!m) return;
    EXPECT(aiq_model_scheme_layers(m) == L && aiq_model_classes(m) == g.classes);
    const int S = 5, N = 7, chunk = 3;
    std::vector<uint8_t> schemes((size_t)S * L);
    for (uint8_t &v : schemes) v = kBits[rng() % 6];
    for (int i = 0; i < L; ++i) schemes[(size_t)1 * L + i] = 32;                             // all-FP32 row
    for (int i = 0; i < L; ++i) schemes[(size_t)2 * L + i] = i == L / 2 ? 4 : schemes[i];     // one layer from row 0
    double ai = 0;
    std::vector<double> fl(n_layers), by(n_layers);
    EXPECT(aiq_layer_ai(g.d.data(), n_layers, schemes.data(), L, 1, fl.data(), by.data(), &ai) == AIQ_OK && ai > 0);
    EXPECT(aiq_layer_ai(g.d.data(), n_layers, schemes.data(), L - 1, 1, nullptr, nullptr, &ai) == AIQ_SHAPE_MISMATCH);

    Buf images(sizeof(float) * g.img_elems * N), top1_base(sizeof(int32_t) * N), agree(sizeof(int32_t) * S);
    Buf logits(sizeof(float) * S * N * g.classes), top1(sizeof(int32_t) * S * N);
    std::memset(images.p, 0, images.n);
    auto f = [](Buf &b) { return static_cast<float *>(b.p); };
    auto i32 = [](Buf &b) { return static_cast<int32_t *>(b.p); };

    for (int shared = 0; shared < 2; ++shared) {
        size_t need = 0;
        st = shared ? aiq_eval_shared_workspace_bytes(m, S, chunk, &need) : aiq_eval_workspace_bytes(m, S, chunk, &need);
        EXPECT(st == AIQ_OK);
        Buf ws(need);
        auto eval = [&](const uint8_t *sch, int s, int n, const uint8_t *ref, int base_valid, float *lg, int32_t *t1,
                        void *wsp, size_t wsb) {
            if (shared)
                return aiq_eval_schemes_shared(m, f(images), n, sch, s, ref, chunk, i32(top1_base), base_valid, lg, t1,
                                               i32(agree), wsp, wsb, nullptr);
            return aiq_eval_schemes(m, f(images), n, sch, s, chunk, i32(top1_base), base_valid, lg, t1, i32(agree), wsp,
                                    wsb, nullptr);
        };
        const std::vector<uint8_t> all32(L, 32);
        const uint8_t *refs[2] = {schemes.data(), all32.data()};
        for (int r = 0; r < (shared ? 2 : 1); ++r)
            for (int base_valid = 0; base_valid < 2; ++base_valid) {
                EXPECT(eval(schemes.data(), S, N, refs[r], base_valid, f(logits), i32(top1), ws.p, need) == AIQ_OK);
                EXPECT(eval(schemes.data(), S, N, refs[r], base_valid, nullptr, nullptr, ws.p, need) == AIQ_OK);
            }
        EXPECT(eval(schemes.data(), 0, N, refs[0], 0, nullptr, nullptr, ws.p, need) == AIQ_OK);
        EXPECT(eval(schemes.data(), S, 0, refs[0], 0, nullptr, nullptr, ws.p, need) == AIQ_OK);
        EXPECT(eval(schemes.data(), 1, 1, refs[0], 0, f(logits), i32(top1), ws.p, need) == AIQ_OK);
        if (need > 1) EXPECT(eval(schemes.data(), S, N, refs[0], 0, nullptr, nullptr, ws.p, need - 1) == AIQ_WORKSPACE_TOO_SMALL);
        EXPECT(eval(schemes.data(), S, N, refs[0], 0, nullptr, nullptr, static_cast<char *>(ws.p) + 16, need) == AIQ_INVALID_ARG);
        std::vector<uint8_t> bad(schemes);
        bad[L + 1 < (int)bad.size() ? L + 1 : 0] = 7;
        EXPECT(eval(bad.data(), S, N, refs[0], 0, nullptr, nullptr, ws.p, need) == AIQ_UNSUPPORTED_BITS);
    }
    {
        size_t need = 0, have = 0;
        EXPECT(aiq_eval_noalloc_workspace_bytes(m, S, chunk, &need, &have) == AIQ_OK && have == AIQ_NOALLOC_SCRATCH_BYTES);
        st = aiq_eval_schemes_noalloc(m, f(images), N, schemes.data(), S, chunk, i32(top1_base), 0, f(logits), i32(top1),
                                      i32(agree), nullptr);
        EXPECT(st == (need <= have ? AIQ_OK : AIQ_WORKSPACE_TOO_SMALL));
    }
    // search drivers and the sensitivity sweep
    aiq_search_params p{};
    p.lambda = 0.9;
    p.n_bits = 3;
    p.bits[0] = 32, p.bits[1] = 8, p.bits[2] = 4;
    p.batch = 1;
    p.max_iters = 2;
    for (int share = 0; share < 2; ++share)
        for (int method = 0; method < 2; ++method) {
            p.share_prefix = share;
            p.only_fp32_layers = method;
            size_t need = 0;
            EXPECT(aiq_search_workspace_bytes(m, N, chunk + 4, 3, &need) == AIQ_OK);
            Buf ws(need);
            std::vector<uint8_t> q(L);
            aiq_search_step trace[4];
            int32_t nt = 0;
            auto fn = method ? aiq_search_greedy : aiq_search_coordinate_descent;
            EXPECT(fn(m, g.d.data(), n_layers, f(images), N, chunk + 4, &p, ws.p, need, nullptr, q.data(), trace, 4, &nt) ==
                   AIQ_OK);
            EXPECT(nt >= 1);
            EXPECT(fn(m, g.d.data(), n_layers, f(images), N, chunk + 4, &p, ws.p, need - 1, nullptr, q.data(), trace, 4,
                      &nt) == AIQ_WORKSPACE_TOO_SMALL);
        }
    {
        const uint8_t bits[2] = {8, 4};
        size_t need = 0;
        EXPECT(aiq_sensitivity_workspace_bytes(m, N, chunk, 2, &need) == AIQ_OK);
        Buf ws(need);
        std::vector<int32_t> out((size_t)L * 2);
        EXPECT(aiq_layer_sensitivity(m, f(images), N, chunk, bits, 2, ws.p, need, nullptr, out.data()) == AIQ_OK);
    }
    // per-kernel timing records
    EXPECT(aiq_profile_enable(m, 1) == AIQ_OK);
    {
        size_t need = 0;
        aiq_eval_workspace_bytes(m, S, chunk, &need);
        Buf ws(need);
        EXPECT(aiq_eval_schemes(m, f(images), N, schemes.data(), S, chunk, i32(top1_base), 0, nullptr, nullptr, i32(agree),
                                ws.p, need, nullptr) == AIQ_OK);
        int64_t launches = 0, total = 0;
        double ms, fl2, by2;
        for (int c = 0; c < AIQ_K_CLASSES; ++c) {
            EXPECT(aiq_profile_read(m, c, &launches, &ms, &fl2, &by2) == AIQ_OK);
            total += launches;
        }
        EXPECT(total > 0);
        EXPECT(aiq_profile_enable(m, 0) == AIQ_OK);
    }
    // one scheme, every node's output (models that run layer by layer)
    {
        const int n_nodes = aiq_model_nodes(m);
        EXPECT(n_nodes == n_layers);
        std::vector<Buf *> outs;
        std::vector<float *> ptrs;
        for (int l = 0; l < n_nodes; ++l) {
            size_t e = 0;
            EXPECT(aiq_node_output_elems(m, l, &e) == AIQ_OK && e > 0);
            outs.push_back(new Buf(sizeof(float) * e * 4));
            ptrs.push_back(static_cast<float *>(outs.back()->p));
        }
        size_t need = 0;
        EXPECT(aiq_eval_workspace_bytes(m, 1, 4, &need) == AIQ_OK);
        Buf ws(need);
        st = aiq_forward_nodes(m, f(images), 4, schemes.data(), ptrs.data(), ws.p, need, nullptr);
        const bool layer_by_layer = (flags & (AIQ_MODEL_LAYERWISE | AIQ_MODEL_ACT_QUANT)) != 0 ||
                                    (!aiq_model_is_lds_resident(m) && aiq_model_lds_resident_blocks(m) == 0);
        EXPECT(layer_by_layer ? (st == AIQ_OK || st == AIQ_UNSUPPORTED_LAYER) : st == AIQ_UNSUPPORTED_LAYER);
        if ((flags & (AIQ_MODEL_LAYERWISE | AIQ_MODEL_ACT_QUANT)) != 0) EXPECT(st == AIQ_OK);
        if (need > 1)
            EXPECT(aiq_forward_nodes(m, f(images), 4, schemes.data(), ptrs.data(), ws.p, need - 1, nullptr) != AIQ_OK);
        for (Buf *b : outs) delete b;
    }
    // deployed inference (models that run layer by layer only; the others are refused)
    for (int variant = 0; variant < 3; ++variant) {
        std::vector<uint8_t> q(L, 8);
        if (variant == 1)
            for (int i = 0; i < L; ++i) q[i] = kBits[rng() % 6];
        aiq_deployed *dep = nullptr;
        st = aiq_deploy_create(m, q.data(), variant == 2 ? AIQ_DEPLOY_FP32_MATRIX : 0, &dep);
        if (aiq_model_is_lds_resident(m) || aiq_model_lds_resident_blocks(m) > 0 ||
            !(flags & (AIQ_MODEL_LAYERWISE | AIQ_MODEL_ACT_QUANT))) {
            if (st != AIQ_OK) {
                EXPECT(st == AIQ_UNSUPPORTED_LAYER && !dep);
                continue;
            }
        }
        EXPECT(st == AIQ_OK && dep);
        if (!dep) continue;
        size_t need = 0;
        EXPECT(aiq_deploy_workspace_bytes(dep, 2, &need) == AIQ_OK);
        Buf ws(need);
        EXPECT(aiq_deploy_forward(dep, f(images), 5, 2, f(logits), i32(top1), ws.p, need, nullptr) == AIQ_OK);
        EXPECT(aiq_deploy_forward(dep, f(images), 5, 2, nullptr, i32(top1), ws.p, need - 1, nullptr) == AIQ_WORKSPACE_TOO_SMALL);
        if (!aiq_model_is_lds_resident(m) && aiq_model_lds_resident_blocks(m) == 0) {
            // every node's output of the deployed scheme, on buffers of exactly the advertised size
            const int nn = aiq_model_nodes(m);
            std::vector<std::unique_ptr<Buf>> outs;
            std::vector<float *> ptrs;
            for (int l = 0; l < nn; ++l) {
                size_t e = 0;
                EXPECT(aiq_node_output_elems(m, l, &e) == AIQ_OK);
                outs.emplace_back(new Buf(e * 3 * sizeof(float)));
                ptrs.push_back(f(*outs.back()));
            }
            size_t need3 = 0;
            EXPECT(aiq_deploy_workspace_bytes(dep, 3, &need3) == AIQ_OK);
            Buf ws3(need3);
            EXPECT(aiq_deploy_forward_nodes(dep, f(images), 3, ptrs.data(), ws3.p, need3, nullptr) == AIQ_OK);
            EXPECT(aiq_deploy_forward_nodes(dep, f(images), 3, ptrs.data(), ws3.p, need3 - 1, nullptr) == AIQ_WORKSPACE_TOO_SMALL);
        }
        aiq_deploy_destroy(dep);
    }
    aiq_model_destroy(m);
}

static void run_oracle(const Graph &g, std::mt19937 &rng, int n_images)
{
    const int n_layers = (int)g.d.size(), L = g.L;
    const int32_t *desc = reinterpret_cast<const int32_t *>(g.d.data());
    EXPECT(oracle_check_graph(desc, n_layers, g.d[0].hin, g.d[0].win, g.d[0].cin) == 0);
    const int S = 2, N = n_images;
    std::vector<uint8_t> schemes((size_t)S * L);
    for (uint8_t &v : schemes) v = kBits[rng() % 6];
    std::vector<float> images(g.img_elems * N);
    std::uniform_real_distribution<float> u(-1.f, 1.f);
    for (float &v : images) v = u(rng);
    std::vector<double> lb((size_t)N * g.classes), lg((size_t)S * N * g.classes);
    std::vector<int32_t> tb(N), t1((size_t)S * N), agree(S);
    for (int per_tensor = 0; per_tensor < 2; ++per_tensor)
        EXPECT(oracle_eval_schemes_ex(desc, n_layers, g.wp.data(), g.bp.data(), images.data(), N, schemes.data(), S, L,
                                      per_tensor, lb.data(), tb.data(), lg.data(), t1.data(), agree.data()) == 0);
    size_t acts = 0;
    for (const aiq_layer_desc &d : g.d)
        acts += d.kind == 2 ? d.cout
                            : (size_t)((d.hin + 2 * d.pad - d.kh) / d.stride + 1) * ((d.win + 2 * d.pad - d.kw) / d.stride + 1) * d.cout;
    std::vector<double> a((size_t)N * acts);
    int64_t macs = 0;
    EXPECT(oracle_forward(desc, n_layers, g.wp.data(), g.bp.data(), images.data(), N, lb.data(), tb.data(), a.data(), &macs) == 0);
    EXPECT(macs > 0);
    double ai = 0;
    std::vector<double> fl(n_layers), by(n_layers);
    EXPECT(oracle_layer_ai(desc, n_layers, schemes.data(), L, 1, fl.data(), by.data(), &ai) == 0 && ai > 0);
    for (int l = 0; l < n_layers; ++l) {
        const aiq_layer_desc &d = g.d[l];
        const int k = (int)(g.w[l].size() / d.cout);
        std::vector<float> dq(g.w[l].size()), sc(d.cout);
        std::vector<int32_t> codes(g.w[l].size());
        for (int bi = 0; bi < 6; ++bi) {
            EXPECT(oracle_quantize_weights(g.w[l].data(), d.cout, k, kBits[bi], dq.data(), sc.data(), codes.data()) == 0);
            EXPECT(oracle_quantize_weights_per_tensor(g.w[l].data(), d.cout, k, kBits[bi], dq.data(), sc.data(), nullptr) == 0);
        }
        EXPECT(oracle_quantize_weights(g.w[l].data(), d.cout, k, 5, dq.data(), sc.data(), nullptr) == 2);
    }
}

int main(int argc, char **argv)
{
    if (argc < 2) return 2;
    std::FILE *fp = std::fopen(argv[1], "rb");
    if (!fp) return 2;
    int32_t n_graphs = 0;
    if (std::fread(&n_graphs, 4, 1, fp) != 1) return 2;
    std::mt19937 rng(12345);
    for (int gi = 0; gi < n_graphs; ++gi) {
        int32_t n = 0, oracle_images = 0;
        if (std::fread(&n, 4, 1, fp) != 1 || std::fread(&oracle_images, 4, 1, fp) != 1) return 2;
        std::vector<int32_t> fields((size_t)n * 13);
        if (std::fread(fields.data(), 4, fields.size(), fp) != fields.size()) return 2;
        Graph g = make_graph(fields.data(), n, rng);
        const long before = aiq_stub_launch_count();
        for (uint32_t flags : {0u, (uint32_t)AIQ_MODEL_LAYERWISE, (uint32_t)AIQ_MODEL_PER_TENSOR,
                               (uint32_t)(AIQ_MODEL_LAYERWISE | AIQ_MODEL_PER_TENSOR), (uint32_t)AIQ_MODEL_ACT_QUANT})
            run_library(g, flags, rng);
        if (oracle_images > 0) run_oracle(g, rng, oracle_images);
        std::printf("graph %d: %d layers, L = %d, %ld launches planned, failures so far %d\n", gi, n, g.L,
                    aiq_stub_launch_count() - before, g_fail);
        std::fflush(stdout);
    }
    std::fclose(fp);
    // argument errors that need no model
    double ai = 0;
    EXPECT(aiq_layer_ai(nullptr, 3, nullptr, 0, 1, nullptr, nullptr, &ai) == AIQ_INVALID_ARG);
    EXPECT(aiq_quantize_weights(nullptr, -1, 4, 8, nullptr, nullptr, nullptr, nullptr) == AIQ_INVALID_ARG);
    EXPECT(aiq_quantize_weights(nullptr, 4, 4, 3, nullptr, nullptr, nullptr, nullptr) == AIQ_UNSUPPORTED_BITS);
    aiq_model *m = nullptr;
    EXPECT(aiq_model_create(nullptr, 0, nullptr, nullptr, &m) == AIQ_INVALID_ARG && !m);
    aiq_model_destroy(nullptr);
    aiq_deploy_destroy(nullptr);
    std::printf(g_fail ? "HOST SANITIZE: %d FAILED\n" : "HOST SANITIZE OK\n", g_fail);
    return g_fail ? 1 : 0;
}
