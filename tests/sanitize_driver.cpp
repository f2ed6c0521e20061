// Host-only driver for the address / undefined-behaviour sanitizer build of the CPU oracle (oracle/lba_ref.cpp)
// and of the host planner (paper_2401_14110_amd/csrc/lba_plan.cpp).  tests/test_sanitizers_cpu.py compiles the
// three files together with -fsanitize=address,undefined -fno-sanitize-recover=all and runs the result; any
// finding of either sanitizer aborts the run.  Nothing here touches a GPU: the planner is plain C++.
//
//   sanitize_driver <roundings file> <chain file>
//     roundings file: lines "x floor rne" of C99 hex floats for Q_acc = M7E4 b=7 (written by the test from
//                     tests/golden/q_m7e4_b7_roundings.txt)
//     chain file:     tests/golden/chain_p1b.txt as it is
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include <vector>

#include "lba_internal.h"

extern "C" {
typedef struct { int32_t exp_bits, man_bits, bias, round; } lba_ref_qfmt;
typedef struct { int32_t exp_bits, man_bits, bias; } lba_ref_infmt;
int lba_ref_gemm(const uint8_t* A, const uint8_t* B, float* C, int64_t M, int64_t N, int64_t K,
                 lba_ref_qfmt qprod, lba_ref_qfmt qacc, int32_t order, int32_t nthreads);
int lba_ref_gemm_bwd(const uint8_t* A, const uint8_t* B, float* C, uint32_t* of_mask, uint32_t* uf_mask,
                     uint32_t* of2_mask, uint32_t* uf2_mask, int64_t M, int64_t N, int64_t K,
                     lba_ref_qfmt qprod, lba_ref_qfmt qacc, int32_t order, int32_t nthreads);
int lba_ref_gemm_diff(const uint8_t* A, const uint8_t* B, float* C, uint32_t* diff_mask, int64_t M, int64_t N, int64_t K,
                      lba_ref_qfmt qprod, lba_ref_qfmt qacc, int32_t order, double eps2, int32_t nthreads);
int lba_ref_gemm_in(const uint8_t* A, const uint8_t* B, float* C, uint32_t* of_mask, uint32_t* uf_mask,
                    int64_t M, int64_t N, int64_t K, lba_ref_infmt fmt_a, lba_ref_infmt fmt_b,
                    lba_ref_qfmt qprod, lba_ref_qfmt qacc, int32_t order, int32_t nthreads);
double lba_ref_decode(uint8_t code);
int lba_ref_quantize(double x, lba_ref_qfmt q, double* out, int32_t* events);
int lba_ref_fmaq(uint8_t a, uint8_t b, double s, lba_ref_qfmt qprod, lba_ref_qfmt qacc, double* out, int32_t* events);
int lba_ref_carrier_bits(lba_ref_qfmt qprod, lba_ref_qfmt qacc);
}

static int failures = 0;
static size_t sz(size_t n) { return n ? n : 1; }   // exact sizes, so that an overrun by one element is seen
#define CHECK(cond, ...) do { if (!(cond)) { std::printf("FAIL %s:%d: ", __FILE__, __LINE__); std::printf(__VA_ARGS__); std::printf("\n"); ++failures; } } while (0)

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd32() {                                      // xorshift64*
    rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
    return (uint32_t)((rng_state * 0x2545F4914F6CDD1Dull) >> 32);
}
static uint8_t rnd_code() {
    uint8_t c = (uint8_t)rnd32();
    if ((c & 0x7F) == 0x7F) c &= 0xFE;                         // no NaN codes
    return c;
}

// 1. the hand-worked roundings of the quantizer (Sec. 2.3), values passed in by the test
static void check_roundings(const char* path) {
    std::FILE* f = std::fopen(path, "r");
    CHECK(f != nullptr, "cannot open %s", path);
    if (!f) return;
    double x, wf, wr;
    int rows = 0;
    while (std::fscanf(f, "%la %la %la", &x, &wf, &wr) == 3) {
        for (int r = 0; r < 2; ++r) {
            lba_ref_qfmt q = {4, 7, 7, r};
            double out = -1.0; int32_t ev = 0;
            CHECK(lba_ref_quantize(x, q, &out, &ev) == 0, "quantize rc");
            CHECK(out == (r ? wr : wf), "Q(%a) round %d: got %a want %a", x, r, out, r ? wr : wf);
        }
        ++rows;
    }
    std::fclose(f);
    CHECK(rows >= 12, "only %d rounding rows", rows);
}

// 2. the hand-worked chain (Sec. 3, App. D): every prefix of it through the GEMM entry point with planes
static void check_chain(const char* path) {
    std::FILE* f = std::fopen(path, "r");
    CHECK(f != nullptr, "cannot open %s", path);
    if (!f) return;
    char line[512];
    std::vector<uint8_t> a, b;
    std::vector<double> sf, sr;
    std::vector<int> off, uff, ofr, ufr;
    while (std::fgets(line, sizeof line, f)) {
        if (line[0] == '#') continue;
        int k, ac, bc, o0, u0, o1, u1; double s0, s1;
        if (std::sscanf(line, "%d %i %i %lf %d %d %lf %d %d", &k, &ac, &bc, &s0, &o0, &u0, &s1, &o1, &u1) == 9) {
            a.push_back((uint8_t)ac); b.push_back((uint8_t)bc); sf.push_back(s0); sr.push_back(s1);
            off.push_back(o0); uff.push_back(u0); ofr.push_back(o1); ufr.push_back(u1);
        }
    }
    std::fclose(f);
    CHECK(a.size() == 4, "chain rows: %zu", a.size());
    for (int r = 0; r < 2; ++r) {
        lba_ref_qfmt qp = {5, 7, 16, r}, qa = {4, 7, 7, r};
        for (size_t K = 1; K <= a.size(); ++K) {
            float C = -1.0f; uint32_t of = ~0u, uf = ~0u;
            CHECK(lba_ref_gemm_bwd(a.data(), b.data(), &C, &of, &uf, nullptr, nullptr, 1, 1, (int64_t)K, qp, qa, 0, 1) == 0, "gemm_bwd rc");
            CHECK((double)C == (r ? sr : sf)[K - 1], "chain K=%zu round %d: %g", K, r, (double)C);
            for (size_t k = 0; k < K; ++k) {
                CHECK((int)((of >> k) & 1u) == (r ? ofr : off)[k], "OF bit %zu K=%zu round %d", k, K, r);
                CHECK((int)((uf >> k) & 1u) == (r ? ufr : uff)[k], "UF bit %zu K=%zu round %d", k, K, r);
            }
            CHECK((of >> K) == 0u && (uf >> K) == 0u, "tail bits");
        }
    }
}

// 3. every entry point of the oracle on ragged shapes, both carriers (128- and 320-bit), both orders, several
//    thread counts: the sanitizers watch the indexing; results must not depend on the thread count
static void run_oracle_entry_points() {
    const int64_t M = 5, N = 3;
    const int64_t Ks[] = {0, 1, 15, 16, 17, 70, 530};
    const lba_ref_qfmt fmts[][2] = {
        {{5, 7, 15, 0}, {4, 7, 7, 0}},   {{5, 7, 15, 1}, {4, 7, 7, 1}},     {{4, 7, 12, 0}, {4, 7, 10, 0}},
        {{5, 3, 15, 1}, {5, 3, 15, 1}},  {{7, 23, 64, 1}, {7, 23, 64, 1}},  {{5, 7, 15, 0x100}, {4, 7, 7, 0x101}},
        {{7, 23, 126, 0}, {2, 1, -124, 0}}, {{2, 1, 126, 1}, {7, 23, 0, 1}}, {{4, 7, 90, 0x100}, {4, 7, 90, 0x100}},
    };
    int wide = 0;
    for (const auto& fm : fmts) {
        const int bits = lba_ref_carrier_bits(fm[0], fm[1]);
        CHECK(bits == 128 || bits == 320, "carrier bits %d", bits);
        wide += bits == 320;
        for (int64_t K : Ks) {
            std::vector<uint8_t> A(sz((size_t)(M * K))), B(sz((size_t)(N * K)));
            for (auto& c : A) c = rnd_code();
            for (auto& c : B) c = rnd_code();
            const size_t W = (size_t)((K + 31) / 32), W2 = (size_t)(((K + 15) / 16 + 31) / 32);
            for (int order = 0; order < 2; ++order) {
                std::vector<float> C1((size_t)(M * N)), C3((size_t)(M * N)), C0((size_t)(M * N));
                std::vector<uint32_t> of1(sz(W * M * N)), uf1(sz(W * M * N)), of3(sz(W * M * N)), uf3(sz(W * M * N));
                std::vector<uint32_t> o2(sz(W2 * M * N)), u2(sz(W2 * M * N)), o23(sz(W2 * M * N)), u23(sz(W2 * M * N));
                CHECK(lba_ref_gemm(A.data(), B.data(), C0.data(), M, N, K, fm[0], fm[1], order, 2) == 0, "gemm rc");
                CHECK(lba_ref_gemm_bwd(A.data(), B.data(), C1.data(), of1.data(), uf1.data(), order ? o2.data() : nullptr,
                                       order ? u2.data() : nullptr, M, N, K, fm[0], fm[1], order, 1) == 0, "bwd rc");
                CHECK(lba_ref_gemm_bwd(A.data(), B.data(), C3.data(), of3.data(), uf3.data(), order ? o23.data() : nullptr,
                                       order ? u23.data() : nullptr, M, N, K, fm[0], fm[1], order, 3) == 0, "bwd rc");
                CHECK(std::memcmp(C0.data(), C1.data(), C0.size() * 4) == 0 && std::memcmp(C1.data(), C3.data(), C1.size() * 4) == 0, "C differs");
                CHECK(std::memcmp(of1.data(), of3.data(), W * M * N * 4) == 0 && std::memcmp(uf1.data(), uf3.data(), W * M * N * 4) == 0, "planes differ");
                if (order) CHECK(std::memcmp(o2.data(), o23.data(), W2 * M * N * 4) == 0 && std::memcmp(u2.data(), u23.data(), W2 * M * N * 4) == 0, "level-2 planes differ");
                std::vector<uint32_t> df(sz(W * M * N));
                // (the two sides of the DIFF comparison need more room: the widest format pairs are refused)
                const int drc = lba_ref_gemm_diff(A.data(), B.data(), C3.data(), df.data(), M, N, K, fm[0], fm[1], order, 0.25, 2);
                CHECK(drc == 0 || bits == 320, "diff rc %d", drc);
                if (drc == 0) CHECK(std::memcmp(C0.data(), C3.data(), C0.size() * 4) == 0, "C of the DIFF call differs");
            }
            const lba_ref_infmt m4e3 = {3, 4, 5}, e5m2 = {5, 2, 15};
            std::vector<float> Ci((size_t)(M * N));
            std::vector<uint32_t> ofi(sz(W * M * N)), ufi(sz(W * M * N));
            if ((fm[0].round & 0x100) == 0)
                CHECK(lba_ref_gemm_in(A.data(), B.data(), Ci.data(), ofi.data(), ufi.data(), M, N, K, m4e3, e5m2, fm[0], fm[1], 0, 2) == 0, "gemm_in rc");
        }
    }
    CHECK(wide >= 2, "no 320-bit case ran");
    // scalar entry points
    for (int i = 0; i < 2000; ++i) {
        lba_ref_qfmt q = {2 + (int)(rnd32() % 6), 1 + (int)(rnd32() % 23), 0, (int)(rnd32() & 1)};
        q.bias = (int)(rnd32() % 60) - 20;
        if ((1 << q.exp_bits) - q.bias - 1 > 127) continue;
        const double x = std::ldexp((double)(int32_t)rnd32(), (int)(rnd32() % 80) - 60);
        double out = 0.0, out2 = 0.0; int32_t ev = 0;
        CHECK(lba_ref_quantize(x, q, &out, &ev) == 0, "quantize rc");
        CHECK(lba_ref_quantize(out, q, &out2, &ev) == 0 && out2 == out, "Q is not idempotent at %a", x);
        lba_ref_qfmt qp = {5, 7, 15, q.round};
        CHECK(lba_ref_fmaq(rnd_code(), rnd_code(), out, qp, q, &out2, &ev) == 0, "fmaq rc");
    }
}

// 4. the planner over the format space, every call kind, both orders, shapes from empty to the documented limits
static void sweep_planner() {
    const int64_t shapes[][3] = {{0, 0, 0}, {1, 1, 1}, {64, 64, 256}, {100352, 64, 576}, {3136, 512, 4608}, {64, 1000, 2048},
                                 {4096, 4096, 4096}, {12544, 1024, 256}, {37, 68, 530}, {(1LL << 30) - 64, 1LL << 21, (1LL << 31) - 64},
                                 {(1LL << 30) - 63, 8, 8}, {8, (1LL << 21) + 1, 8}, {-1, 8, 8}, {200704, 256, 64}, {802816, 64, 147}};
    const int mans[] = {1, 3, 6, 7, 8, 10, 11, 21, 22, 23};
    const int rounds[] = {0, 1, 0x100, 0x101, 2, 0x200};
    long plans = 0, fast = 0, mixed = 0;
    for (const auto& sh : shapes)
        for (int Ep = 2; Ep <= 7; Ep += 1)
            for (int Ea = 2; Ea <= 7; ++Ea)
                for (int mp : {4, 7, 12})
                    for (int ma : mans)
                        for (int bi = 0; bi < 5; ++bi)
                            for (int r : rounds)
                                for (int order = 0; order <= 2; ++order)
                                    for (int events = 0; events <= 3; ++events) {
                                        const int lo_p = (1 << Ep) - 128, lo_a = (1 << Ea) - 128;
                                        const int bp = bi == 0 ? lo_p - 1 : bi == 1 ? lo_p : bi == 2 ? 15 : bi == 3 ? 126 : 127;
                                        const int ba = bi == 0 ? lo_a : bi == 1 ? 7 : bi == 2 ? -9 : bi == 3 ? 90 : 126;
                                        const lba_qfmt qp = {Ep, mp, bp, r & 0x1FF}, qa = {Ea, ma, ba, r};
                                        lba::Plan pl;
                                        const int rc = lba::make_plan(sh[0], sh[1], sh[2], qp, qa, order, events, &pl);
                                        CHECK(rc >= LBA_OK && rc <= LBA_ERR_LAUNCH, "status %d", rc);
                                        if (rc != LBA_OK) continue;
                                        ++plans;
                                        const int64_t M = sh[0], N = sh[1];
                                        CHECK(pl.kernel == lba::KERNEL_FAST || pl.kernel == lba::KERNEL_GEN, "kernel %d", pl.kernel);
                                        CHECK(pl.bk == 32 && (pl.tm == 2 || pl.tm == 4) && (pl.tn == 2 || pl.tn == 4), "tile");
                                        if (pl.mix_tail > 0) {
                                            ++mixed;
                                            const lba::KParams& kp = pl.kp;
                                            const int64_t gy64 = (N + 63) / 64, gy32 = (N + 31) / 32;
                                            CHECK(kp.mix_m_main % 64 == 0 && kp.mix_m_main <= M && kp.mix_main == kp.mix_m_main / 64 * gy64, "64-row region");
                                            CHECK(kp.mix_main == 0 || kp.mix_m_main == (int64_t)kp.mix_gx_main * 64, "64-row region width");
                                            CHECK(kp.mix_m_half >= kp.mix_m_main && kp.mix_m_half <= M && (kp.mix_m_half - kp.mix_m_main) % 48 == 0, "48-row region");
                                            CHECK(kp.mix_half == (kp.mix_m_half - kp.mix_m_main) / 48 * gy64, "48-row count");
                                            CHECK(kp.mix_half == 0 || kp.mix_m_half - kp.mix_m_main == (int64_t)kp.mix_gx_half * 48, "48-row region width");
                                            CHECK(kp.mix_half == 0 || events == 0, "48-row tiles are the forward kernel's");
                                            const int64_t quarters = pl.mix_tail - kp.mix_half;
                                            CHECK(quarters >= 0 && (quarters == 0) == (kp.mix_m_half >= M), "32-row region present iff rows are left");
                                            CHECK(quarters == 0 || ((int64_t)kp.mix_gx_tail * 32 >= M - kp.mix_m_half && (int64_t)(kp.mix_gx_tail - 1) * 32 < M - kp.mix_m_half), "tail rows cover M");
                                            CHECK(quarters == 0 || quarters == kp.mix_gx_tail * (kp.mix_tail16 ? (N + 15) / 16 : gy32), "tail count");
                                            CHECK(kp.mix_tail16 == 0 || (events == 0 && kp.mix_gx_tail * gy32 <= 128 && kp.mix_main + kp.mix_half >= 0 &&
                                                                         (kp.mix_main + kp.mix_half) % 1024 == 0), "32 x 16 tail only where it runs alone");
                                            CHECK(kp.mix_gx_main >= 1 && kp.mix_gx_half >= 1 && kp.mix_gx_tail >= 1, "divisors");
                                            CHECK(pl.grid_x == kp.mix_main + pl.mix_tail && pl.grid_y == 1, "mixed grid");
                                        } else if (pl.kpar > 0) {
                                            const int64_t tm = pl.kpar == 1 ? 32 : 8, tn = pl.kpar == 1 ? 32 : 16;
                                            CHECK(pl.kpar == 1 || pl.kpar == 3, "kpar %d", pl.kpar);
                                            CHECK(order == LBA_ORDER_CHUNK16 && events == 0 && pl.kernel == lba::KERNEL_FAST, "kpar plan");
                                            CHECK(pl.grid_x * tm >= M && pl.grid_y * tn >= N && (pl.grid_x - 1) * tm < M && (pl.grid_y - 1) * tn < N, "kpar grid");
                                            CHECK(pl.grid_y <= 65535 && (int64_t)pl.grid_x * pl.grid_y >= 1, "kpar grid limits");
                                        } else {
                                            CHECK((int64_t)pl.grid_x * 16 * pl.tm >= M && (int64_t)pl.grid_y * 16 * pl.tn >= N, "grid covers the outputs");
                                            CHECK((int64_t)(pl.grid_x - 1) * 16 * pl.tm < M || M == 0, "no empty tile row");
                                        }
                                        if (pl.kernel == lba::KERNEL_FAST) {
                                            ++fast;
                                            CHECK(pl.valu_per_mac_x100 >= 200, "slots %d", pl.valu_per_mac_x100);
                                            CHECK(std::isnormal(pl.kp.kc) && std::isnormal(pl.kp.rof_a), "kc %a rof %a", (double)pl.kp.kc, (double)pl.kp.rof_a);
                                        } else {
                                            CHECK(std::isnormal(pl.kp.rof_a) && std::isnormal(pl.kp.rof_p), "general kernel: R_OF not a normal");
                                        }
                                    }
    CHECK(plans > 100000 && fast > 1000 && mixed > 100, "sweep too small: %ld plans, %ld fast, %ld mixed", plans, fast, mixed);
    // operand-format specs and the gradient split
    for (int ea = 1; ea <= 6; ++ea)
        for (int eb = 1; eb <= 6; ++eb)
            for (int b : {-33, -32, 0, 7, 32, 33}) {
                lba::InSpec s;
                const lba_infmt fa = {ea, 7 - ea, b}, fb = {eb, 7 - eb, -b};
                const int rc = lba::make_in_spec(fa, fb, &s);
                const bool ok = ea >= 2 && ea <= 5 && eb >= 2 && eb <= 5 && b >= -32 && b <= 32;
                CHECK((rc == LBA_OK) == ok, "in-spec %d %d %d: %d", ea, eb, b, rc);
                if (rc == LBA_OK) {
                    lba::Plan pl;
                    const lba_qfmt qp = {5, 7, 15, 0}, qa = {4, 7, 7, 0};
                    CHECK(lba::make_plan(300, 70, 90, qp, qa, 0, 0, &pl, 1, &s) == LBA_OK, "plan with in-spec");
                }
            }
    for (int64_t blocks : {1LL, 3LL, 100LL, 1024LL, 5000LL, 1LL << 30})
        for (int64_t S : {1LL, 4LL, 63LL, 64LL, 1000LL, 4096LL, 1LL << 30}) {
            int split = 0; int32_t chunk = 0;
            lba::plan_grad_split(blocks, S, &split, &chunk);
            CHECK(split >= 1 && split <= 65535 && chunk >= 4 && chunk % 4 == 0 && (int64_t)split * chunk >= S, "split %d chunk %d", split, chunk);
        }
}

int main(int argc, char** argv) {
    if (argc != 3) { std::printf("usage: %s <roundings> <chain>\n", argv[0]); return 2; }
    check_roundings(argv[1]);
    check_chain(argv[2]);
    run_oracle_entry_points();
    sweep_planner();
    if (failures) { std::printf("%d failures\n", failures); return 1; }
    std::printf("sanitize driver ok\n");
    return 0;
}
