// Host-only exercise of the C ABI under AddressSanitizer / UndefinedBehaviorSanitizer: the packing step, the
// wavefront scheduler, every argument / shape / workspace error path that is reported before a launch, and the
// section executor's plan and sequencing with the kernels replaced by the stand-ins of fake_backend.cpp.  Every
// buffer is allocated at exactly its documented size, so any out-of-bounds carve-out or mis-sized argument is a
// sanitizer report (the process then exits non-zero).
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <map>
#include <memory>
#include <random>
#include <string>
#include <vector>

#include "maestro_kernels.h"
#include "maestro_section.h"

extern std::map<std::string, long> g_calls;
static int g_checks = 0;
constexpr int kKdStatFloats = 8;   // per-token statistics the KD step keeps (documented workspace layout)
#define CHECK(cond)                                                                              \
    do {                                                                                         \
        ++g_checks;                                                                              \
        if (!(cond)) { fprintf(stderr, "FAILED %s:%d: %s  [%s]\n", __FILE__, __LINE__, #cond, ms_last_error()); exit(1); } \
    } while (0)

struct Buf {   // exact-size heap block (so the sanitizer sees its true bounds)
    void *p;
    size_t n;
    explicit Buf(size_t bytes) : p(bytes ? malloc(bytes) : nullptr), n(bytes) { if (p) memset(p, 1, bytes); }
    ~Buf() { free(p); }
    Buf(const Buf &) = delete;
};

static void test_pack(std::mt19937 &rng) {
    for (int trial = 0; trial < 200; ++trial) {
        const int n = rng() % 40;
        std::vector<int32_t> len(n), order(n ? n : 1), offs(n + 1), cu(2 * n ? 2 * n : 1);
        for (auto &l : len) l = (rng() % 4 == 0) ? 0 : rng() % 300;
        const int budget = 1 + rng() % 500, policy = rng() % 2;
        int32_t n_mb = -1;
        CHECK(ms_pack_microbatches(len.data(), n, budget, policy, order.data(), offs.data(), &n_mb, cu.data()) == MS_OK);
        CHECK(n_mb >= 0 && n_mb <= n && offs[0] == 0);
        long kept = 0;
        for (int l : len) kept += l > 0;
        CHECK(offs[n_mb] == kept);
        int pos = 0;
        for (int m = 0; m < n_mb; ++m) {                       // each micro-batch: a prefix sum from 0 within the budget
            CHECK(cu[pos] == 0);
            const int k = offs[m + 1] - offs[m];
            for (int i = 0; i < k; ++i) CHECK(cu[pos + i + 1] - cu[pos + i] == len[order[offs[m] + i]]);
            CHECK(k == 1 || cu[pos + k] <= budget);
            pos += k + 1;
        }
    }
    int32_t one = 5, o, off[2], cu[2], nmb;
    CHECK(ms_pack_microbatches(&one, 1, 0, 0, &o, off, &nmb, cu) == MS_ERR_INVALID_ARG);
    CHECK(ms_pack_microbatches(&one, 1, 8, 2, &o, off, &nmb, cu) == MS_ERR_INVALID_ARG);
    CHECK(ms_pack_microbatches(nullptr, 1, 8, 0, &o, off, &nmb, cu) == MS_ERR_INVALID_ARG);
    int32_t neg = -1;
    CHECK(ms_pack_microbatches(&neg, 1, 8, 0, &o, off, &nmb, cu) == MS_ERR_INVALID_ARG);
    CHECK(ms_pack_microbatches(nullptr, 0, 8, 0, nullptr, off, &nmb, nullptr) == MS_OK && nmb == 0);
}

static void test_schedule(std::mt19937 &rng) {
    std::uniform_real_distribution<double> u(0.0, 3.0);
    for (int n : {0, 1, 2, 5, 17, 64}) {
        for (int interleave = 0; interleave < 2; ++interleave) {
            std::vector<double> t(6 * n ? 6 * n : 1);
            for (auto &v : t) v = (rng() % 5 == 0) ? 0.0 : u(rng);
            std::vector<int32_t> order(n ? n : 1);
            double mk = -1, mk2 = -1, idle = -1;
            CHECK(ms_schedule_samples(n, t.data(), interleave, order.data(), &mk) == MS_OK);
            std::vector<char> seen(n, 0);
            for (int i = 0; i < n; ++i) { CHECK(order[i] >= 0 && order[i] < n && !seen[order[i]]); seen[order[i]] = 1; }
            CHECK(ms_schedule_makespan(n, t.data(), order.data(), interleave, &mk2, &idle) == MS_OK);
            CHECK(mk2 <= mk * (1 + 1e-9) + 1e-12 && mk <= mk2 * (1 + 1e-9) + 1e-12 && idle >= -1e-12);
            if (n >= 2) {
                order[0] = order[1];                            // not a permutation
                CHECK(ms_schedule_makespan(n, t.data(), order.data(), interleave, &mk2, nullptr) == MS_ERR_INVALID_ARG);
            }
        }
    }
    double bad[6] = {1, 1, 1, -1, 1, 1};
    int32_t o;
    CHECK(ms_schedule_samples(1, bad, 1, &o, nullptr) == MS_ERR_INVALID_ARG);
    CHECK(ms_schedule_samples(-1, bad, 1, &o, nullptr) == MS_ERR_INVALID_ARG);
}

struct SectionCase {
    ms_section_config c;
    std::vector<int32_t> cu;
};

// Runs ms_section_forward and ms_section_forward_backward (both gradient sources) on exact-size buffers.
static void run_section(const SectionCase &sc, bool with_kd) {
    const ms_section_config &c = sc.c;
    const size_t es = c.dtype == MS_BF16 ? 2 : 4;
    const int n = sc.cu.back(), n_seqs = (int)sc.cu.size() - 1;
    int max_seqlen = 0;
    for (int i = 0; i < n_seqs; ++i) max_seqlen = std::max(max_seqlen, sc.cu[i + 1] - sc.cu[i]);
    const int d = c.d_model, dqkv = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim, dattn = c.n_q_heads * c.head_dim;
    const int dup = c.arch == MS_DECODER ? 2 * c.d_ffn : c.d_ffn;
    const bool enc = c.arch == MS_ENCODER;
    // weights (storage type) and gradients (fp32), each tensor its own exact-size block
    std::vector<std::unique_ptr<Buf>> keep;
    auto blk = [&](size_t bytes) { keep.emplace_back(new Buf(bytes)); return keep.back()->p; };
    std::vector<ms_layer_ptrs> wl(c.n_layers), gl(c.n_layers);
    auto fill_layer = [&](ms_layer_ptrs &l, size_t e) {
        l.norm1_g = blk(d * e); l.norm1_b = enc ? blk(d * e) : nullptr;
        l.w_qkv = blk((size_t)dqkv * d * e); l.b_qkv = enc ? blk(dqkv * e) : nullptr;
        l.w_o = blk((size_t)d * dattn * e); l.b_o = enc ? blk(d * e) : nullptr;
        l.norm2_g = blk(d * e); l.norm2_b = enc ? blk(d * e) : nullptr;
        l.w_up = blk((size_t)dup * d * e); l.b_up = enc ? blk(dup * e) : nullptr;
        l.w_down = blk((size_t)d * c.d_ffn * e); l.b_down = enc ? blk(d * e) : nullptr;
    };
    for (auto &l : wl) fill_layer(l, es);
    for (auto &l : gl) fill_layer(l, 4);
    ms_section_ptrs w = {c.vocab ? blk((size_t)c.vocab * d * es) : nullptr, wl.data(), blk(d * es), enc ? blk(d * es) : nullptr};
    ms_section_ptrs g = {c.vocab ? blk((size_t)c.vocab * d * 4) : nullptr, gl.data(), blk(d * 4), enc ? blk(d * 4) : nullptr};
    Buf cu_dev(sc.cu.size() * 4);
    memcpy(cu_dev.p, sc.cu.data(), sc.cu.size() * 4);
    ms_batch b = {n, n_seqs, (const int32_t *)cu_dev.p, sc.cu.data()};
    Buf x_in(c.vocab ? (size_t)n * 4 : (size_t)n * d * es), h_out((size_t)n * d * es);
    // ---- forward only
    const size_t need_f = ms_section_workspace_bytes(&c, n, max_seqlen, 0);
    CHECK(need_f > 0);
    {
        Buf ws(need_f);
        CHECK(ms_section_forward(&c, &w, &b, x_in.p, h_out.p, ws.p, ws.n, nullptr) == MS_OK);
        CHECK(ms_section_forward(&c, &w, &b, x_in.p, h_out.p, ws.p, ws.n - 1, nullptr) == MS_ERR_WORKSPACE);
        CHECK(ms_section_forward(&c, &w, &b, nullptr, h_out.p, ws.p, ws.n, nullptr) == MS_ERR_INVALID_ARG);
    }
    // ---- forward + backward from an upstream gradient
    const size_t need_b = ms_section_workspace_bytes(&c, n, max_seqlen, 1);
    CHECK(need_b >= need_f);
    Buf d_h((size_t)n * d * es), d_x(c.vocab ? 0 : (size_t)n * d * es);
    {
        Buf ws(need_b);
        const long gemms = g_calls["gemm"] + g_calls["gemm_swiglu"];
        CHECK(ms_section_forward_backward(&c, &w, &g, &b, x_in.p, h_out.p, d_h.p, nullptr, nullptr, nullptr, nullptr, nullptr,
                                          d_x.p, ws.p, ws.n, nullptr) == MS_OK);
        // per layer 4 forward linears, 4 input-gradient and 4 weight-gradient products
        CHECK(g_calls["gemm"] + g_calls["gemm_swiglu"] - gemms == 12L * c.n_layers);
        CHECK(ms_section_forward_backward(&c, &w, &g, &b, x_in.p, h_out.p, d_h.p, nullptr, nullptr, nullptr, nullptr, nullptr,
                                          d_x.p, ws.p, ws.n - 1, nullptr) == MS_ERR_WORKSPACE);
        CHECK(ms_section_forward_backward(&c, &w, &g, &b, x_in.p, h_out.p, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                          d_x.p, ws.p, ws.n, nullptr) == MS_ERR_INVALID_ARG);      // no gradient source
    }
    // ---- forward + backward with the KD loss attached
    if (with_kd) {
        const int V = 520, Ht = 48;
        Buf wt((size_t)V * Ht * es), wsd((size_t)V * d * es), h_t((size_t)n * Ht * es), d_ws((size_t)V * d * 4), loss(4), kl((size_t)n * 4);
        ms_kd_config kd = {V, Ht, d, 128, c.dtype, 2.f, 1.f / n, wt.p, wsd.p, 0};
        const size_t need_kd = ms_kd_workspace_bytes(&kd, n);
        CHECK(need_kd > 0);
        Buf ws(need_b + need_kd);
        CHECK(ms_section_forward_backward(&c, &w, &g, &b, x_in.p, h_out.p, nullptr, &kd, h_t.p, d_ws.p, (float *)loss.p,
                                          (float *)kl.p, d_x.p, ws.p, ws.n, nullptr) == MS_OK);
        CHECK(ms_section_forward_backward(&c, &w, &g, &b, x_in.p, h_out.p, nullptr, &kd, h_t.p, d_ws.p, (float *)loss.p,
                                          (float *)kl.p, d_x.p, ws.p, ws.n - 1, nullptr) == MS_ERR_WORKSPACE);
        CHECK(ms_section_forward_backward(&c, &w, &g, &b, x_in.p, h_out.p, d_h.p, &kd, h_t.p, d_ws.p, (float *)loss.p,
                                          (float *)kl.p, d_x.p, ws.p, ws.n, nullptr) == MS_ERR_INVALID_ARG);   // two sources
        ms_kd_config bad = kd;
        bad.h_student = d + 8;
        CHECK(ms_section_forward_backward(&c, &w, &g, &b, x_in.p, h_out.p, nullptr, &bad, h_t.p, d_ws.p, (float *)loss.p,
                                          (float *)kl.p, d_x.p, ws.p, ws.n, nullptr) == MS_ERR_SHAPE);
        CHECK(ms_section_forward_backward(&c, &w, &g, &b, x_in.p, h_out.p, nullptr, &kd, h_t.p, d_ws.p, nullptr,
                                          (float *)kl.p, d_x.p, ws.p, ws.n, nullptr) == MS_ERR_INVALID_ARG);   // no loss_dev
    }
    // ---- the skipped-section case launches nothing and needs nothing
    int32_t cu0[2] = {0, 0};
    ms_batch empty = {0, 1, nullptr, cu0};
    const long before = g_calls["gemm"];
    CHECK(ms_section_forward(&c, &w, &empty, nullptr, nullptr, nullptr, 0, nullptr) == MS_OK && g_calls["gemm"] == before);
}

static void test_sections() {
    const ms_section_config dec_bf16 = {MS_DECODER, MS_BF16, 2, 128, 4, 2, 64, 192, 96, 1e-6f, 1e4f};     // K % 64 == 0: fused SwiGLU path
    const ms_section_config dec_bf16_odd = {MS_DECODER, MS_BF16, 1, 72, 3, 1, 80, 104, 0, 1e-6f, 1e4f};  // unfused path, embeddings in
    const ms_section_config dec_f32 = {MS_DECODER, MS_F32, 1, 64, 2, 2, 64, 88, 40, 1e-6f, 1e4f};
    const ms_section_config enc_bf16 = {MS_ENCODER, MS_BF16, 2, 80, 2, 2, 128, 160, 0, 1e-6f, 0.f};
    run_section({dec_bf16, {0, 5, 5, 21, 30}}, true);
    run_section({dec_bf16_odd, {0, 17}}, true);
    run_section({dec_f32, {0, 3, 11}}, true);
    run_section({enc_bf16, {0, 9, 40}}, false);
    CHECK(g_calls["gemm_swiglu"] > 0 && g_calls["act_forward"] > 0 && g_calls["colsum"] > 0 && g_calls["kd"] == 3);

    // ---- configuration and batch errors, all before any launch (the pointers below are never dereferenced)
    ms_layer_ptrs lp = {};
    ms_section_ptrs w = {nullptr, &lp, nullptr, nullptr};
    int32_t cu[3] = {0, 4, 8};
    ms_batch b = {8, 2, cu, cu};
    char dummy[8];
    auto fwd = [&](ms_section_config c, const ms_batch *bb = nullptr) {
        return ms_section_forward(&c, &w, bb ? bb : &b, dummy, dummy, dummy, 8, nullptr);
    };
    ms_section_config c = dec_bf16;
    CHECK(ms_section_forward(nullptr, &w, &b, dummy, dummy, dummy, 8, nullptr) == MS_ERR_INVALID_ARG);
    c = dec_bf16; c.arch = 7; CHECK(fwd(c) == MS_ERR_INVALID_ARG);
    c = dec_bf16; c.dtype = 3; CHECK(fwd(c) == MS_ERR_INVALID_ARG);
    c = dec_bf16; c.n_layers = 0; CHECK(fwd(c) == MS_ERR_SHAPE);
    c = dec_bf16; c.n_kv_heads = 3; CHECK(fwd(c) == MS_ERR_SHAPE);
    c = dec_bf16; c.head_dim = 96; CHECK(fwd(c) == MS_ERR_UNSUPPORTED);
    c = dec_bf16; c.d_model = 100; CHECK(fwd(c) == MS_ERR_UNSUPPORTED);
    c = dec_bf16; c.rope_base = 0.5f; CHECK(fwd(c) == MS_ERR_INVALID_ARG);
    c = dec_bf16; c.norm_eps = -1.f; CHECK(fwd(c) == MS_ERR_INVALID_ARG);
    CHECK(ms_section_workspace_bytes(&c, 8, 8, 0) == 0);
    int32_t cu_dec[3] = {0, 5, 4}, cu_end[3] = {0, 4, 7}, cu_start[3] = {1, 4, 8};
    ms_batch bad = b;
    bad.cu_seqlens_host = cu_dec; CHECK(fwd(dec_bf16, &bad) == MS_ERR_INVALID_ARG);
    bad.cu_seqlens_host = cu_end; CHECK(fwd(dec_bf16, &bad) == MS_ERR_INVALID_ARG);
    bad.cu_seqlens_host = cu_start; CHECK(fwd(dec_bf16, &bad) == MS_ERR_INVALID_ARG);
    bad = b; bad.cu_seqlens_dev = nullptr; CHECK(fwd(dec_bf16, &bad) == MS_ERR_INVALID_ARG);
    bad = b; bad.n_tokens = -1; CHECK(fwd(dec_bf16, &bad) == MS_ERR_INVALID_ARG);
    CHECK(fwd(dec_bf16) == MS_ERR_INVALID_ARG);                   // null weight pointers inside the layer
    // kernel limits are part of the up-front checks: a batch beyond the attention kernels' 4 GiB of qkv ...
    int32_t cu_big[2] = {0, 6000000};
    ms_batch big = {6000000, 1, cu, cu_big};
    CHECK(fwd(dec_bf16, &big) == MS_ERR_UNSUPPORTED && strstr(ms_last_error(), "4 GiB"));
    // ... and a model wider than the norm backward kernel holds (only when a backward pass is asked for)
    c = dec_bf16; c.d_model = 8192;
    CHECK(ms_section_forward_backward(&c, &w, &w, &b, dummy, dummy, dummy, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                      dummy, 8, nullptr) == MS_ERR_UNSUPPORTED && strstr(ms_last_error(), "norm backward"));
    CHECK(fwd(c) == MS_ERR_INVALID_ARG);                          // forward only: passes the limit, stops at the null weights
}

static void test_kd() {
    // the KD configuration is validated by the section call it is attached to, before anything else of the call runs
    char dummy[8];
    const ms_section_config sc = {MS_DECODER, MS_BF16, 1, 128, 2, 2, 64, 192, 0, 1e-6f, 1e4f};
    ms_layer_ptrs lp = {};
    ms_section_ptrs w = {nullptr, &lp, nullptr, nullptr};
    int32_t cu[2] = {0, 16};
    ms_batch b = {16, 1, cu, cu};
    ms_kd_config kd = {1024, 256, 128, 256, MS_BF16, 2.f, 1.f, dummy, dummy, 0};
    CHECK(ms_kd_workspace_bytes(&kd, 100) > 0 && ms_kd_workspace_bytes(nullptr, 100) == 0 && ms_kd_workspace_bytes(&kd, -1) == 0);
    auto call = [&](ms_kd_config k) {
        return ms_section_forward_backward(&sc, &w, &w, &b, dummy, dummy, nullptr, &k, dummy, dummy, (float *)dummy, nullptr, nullptr,
                                           dummy, 8, nullptr);
    };
    ms_kd_config k = kd;
    k.dtype = 5; CHECK(call(k) == MS_ERR_INVALID_ARG);
    k = kd; k.vocab = 0; CHECK(call(k) == MS_ERR_SHAPE);
    k = kd; k.temperature = 0.f; CHECK(call(k) == MS_ERR_INVALID_ARG);
    k = kd; k.token_block = 12; CHECK(call(k) == MS_ERR_INVALID_ARG);
    k = kd; k.chunk = 100; CHECK(call(k) == MS_ERR_UNSUPPORTED);
    k = kd; k.w_student_dev = nullptr; CHECK(call(k) == MS_ERR_INVALID_ARG);
    CHECK(call(kd) == MS_ERR_INVALID_ARG && strstr(ms_last_error(), "null"));      // valid KD config: stops at the null weights
    // token-block variant: the cache grows with the vocabulary, not with the token count
    k = kd; k.token_block = 64;
    CHECK(ms_kd_workspace_bytes(&k, 64) > ms_kd_workspace_bytes(&kd, 64));
    CHECK(ms_kd_workspace_bytes(&k, 64 * 50) - ms_kd_workspace_bytes(&k, 64) ==
          (size_t)64 * 49 * (kKdStatFloats * 4 + 128 * 4));                      // only statistics and the dHs accumulator grow
}

int main() {
    std::mt19937 rng(12345);
    test_pack(rng);
    test_schedule(rng);
    test_sections();
    test_kd();
    printf("host sanitizer driver: OK (%d checks)\n", g_checks);
    return 0;
}
