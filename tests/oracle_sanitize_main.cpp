// Driver for the sanitizer build of the CPU oracle and of the library's host-only code
// (chunk scheduler): compiled by tests/test_sanitizers_cpu.py with
// -fsanitize=address,undefined and run as a child process.  It calls the oracle on
// shapes that reach every loop tail (row blocks with a remainder, fewer than four rows,
// selections, no valid row) and checks properties that hold for any input, so that a
// run is more than a smoke test; exit status 0 = everything held and no sanitizer report.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "scheduler.h"

extern "C" {
int flce_oracle_f64(const double* X, const double* W, const int64_t* targets, int64_t BT, int64_t H,
                    int64_t V, int64_t ignore_index, const int64_t* rows_sel, int64_t n_rows_sel,
                    const int64_t* vocab_sel, int64_t n_vocab_sel, double* loss, double* lse,
                    double* dX, double* dW, double* G);
int flce_oracle_f32in(const float* X, const float* W, const int64_t* targets, int64_t BT, int64_t H,
                      int64_t V, int64_t ignore_index, const int64_t* rows_sel, int64_t n_rows_sel,
                      const int64_t* vocab_sel, int64_t n_vocab_sel, double* loss, double* lse,
                      double* dX, double* dW, double* G);
int ce_oracle_f64(double* z, const int64_t* targets, int64_t BT, int64_t V, int64_t ignore_index,
                  double* loss, double* lse);
}

static int failures = 0;
#define CHECK(cond, ...)                                   \
    do {                                                   \
        if (!(cond)) {                                     \
            std::printf("FAILED %s:%d: ", __FILE__, __LINE__); \
            std::printf(__VA_ARGS__);                      \
            std::printf("\n");                             \
            ++failures;                                    \
        }                                                  \
    } while (0)

static uint64_t rng_state = 88172645463325252ull;
static double uniform() {   // xorshift64, enough for test inputs
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0;
}

static void oracle_case(int64_t BT, int64_t H, int64_t V, int every_nth_ignored, bool zero_w) {
    const int64_t IGN = -100;
    std::vector<double> X(BT * H), W(V * H);
    std::vector<float> Xf(BT * H), Wf(V * H);
    for (size_t i = 0; i < X.size(); ++i) X[i] = Xf[i] = (float)(2.0 * uniform() - 1.0);
    for (size_t i = 0; i < W.size(); ++i) W[i] = Wf[i] = zero_w ? 0.f : (float)(0.2 * uniform() - 0.1);
    std::vector<int64_t> t(BT);
    int64_t n_valid = 0;
    for (int64_t i = 0; i < BT; ++i) {
        const bool ign = every_nth_ignored == 1 || (every_nth_ignored > 1 && i % every_nth_ignored == 0);
        t[i] = ign ? IGN : (int64_t)(uniform() * V) % V;
        n_valid += !ign;
    }
    double loss = -1.0;
    std::vector<double> lse(BT), dX(BT * H), dW(V * H), G(BT * V);
    int rc = flce_oracle_f64(X.data(), W.data(), t.data(), BT, H, V, IGN, nullptr, 0, nullptr, 0, &loss,
                             lse.data(), dX.data(), dW.data(), G.data());
    CHECK(rc == 0, "oracle rc %d", rc);
    for (int64_t i = 0; i < BT; ++i) {   // rows of dlogits sum to zero; ignored rows are zero
        double s = 0.0, a = 0.0;
        for (int64_t v = 0; v < V; ++v) {
            s += G[i * V + v];
            a += std::fabs(G[i * V + v]);
        }
        CHECK(std::fabs(s) <= 1e-14, "row %lld of dlogits sums to %g", (long long)i, s);
        if (t[i] == IGN) {
            CHECK(a == 0.0, "ignored row %lld has dlogits", (long long)i);
            for (int64_t h = 0; h < H; ++h) CHECK(dX[i * H + h] == 0.0, "ignored row has dX");
        }
    }
    for (int64_t h = 0; h < H; ++h) {    // hence the columns of dW sum to zero
        double s = 0.0, a = 0.0;
        for (int64_t v = 0; v < V; ++v) {
            s += dW[v * H + h];
            a += std::fabs(dW[v * H + h]);
        }
        CHECK(std::fabs(s) <= 1e-13 * (1.0 + a), "column %lld of dW sums to %g", (long long)h, s);
    }
    if (n_valid == 0) CHECK(loss == 0.0, "loss without valid rows is %g", loss);
    if (zero_w && n_valid > 0)
        CHECK(std::fabs(loss - std::log((double)V)) <= 1e-12, "W = 0: loss %g, log V %g", loss,
              std::log((double)V));

    // selections are slices of the full result, and fp32-held inputs widen exactly
    std::vector<int64_t> rows = {BT - 1, 0, BT / 2}, vocab = {V - 1, 0, V / 3};
    std::vector<double> dXs(rows.size() * H), dWs(vocab.size() * H);
    double loss2 = -1.0;
    rc = flce_oracle_f32in(Xf.data(), Wf.data(), t.data(), BT, H, V, IGN, rows.data(),
                           (int64_t)rows.size(), vocab.data(), (int64_t)vocab.size(), &loss2, nullptr,
                           dXs.data(), dWs.data(), nullptr);
    CHECK(rc == 0 && loss2 == loss, "fp32-held inputs: rc %d loss %g vs %g", rc, loss2, loss);
    for (size_t j = 0; j < rows.size(); ++j)
        for (int64_t h = 0; h < H; ++h)
            CHECK(dXs[j * H + h] == dX[rows[j] * H + h], "selected dX row differs");
    for (size_t j = 0; j < vocab.size(); ++j)
        for (int64_t h = 0; h < H; ++h)
            CHECK(dWs[j * H + h] == dW[vocab[j] * H + h], "selected dW row differs");

    // a target outside [0, V) is rejected, nothing is written past the arrays
    if (BT > 0) {
        std::vector<int64_t> bad(t);
        bad[BT - 1] = V;
        rc = flce_oracle_f64(X.data(), W.data(), bad.data(), BT, H, V, IGN, nullptr, 0, nullptr, 0, &loss2,
                             nullptr, nullptr, nullptr, nullptr);
        CHECK(rc == 2, "out-of-range target accepted (rc %d)", rc);
    }

    // stand-alone cross entropy on the same logits gives the same dlogits
    std::vector<double> Z(BT * V);
    for (int64_t i = 0; i < BT; ++i)
        for (int64_t v = 0; v < V; ++v) {
            double acc = 0.0;
            for (int64_t k = 0; k < H; ++k) acc += X[i * H + k] * W[v * H + k];
            Z[i * V + v] = acc;
        }
    double loss3 = -1.0;
    rc = ce_oracle_f64(Z.data(), t.data(), BT, V, IGN, &loss3, nullptr);
    CHECK(rc == 0 && std::fabs(loss3 - loss) <= 1e-12 * (1.0 + std::fabs(loss)), "CE loss %g vs %g", loss3,
          loss);
    double worst = 0.0;
    for (size_t i = 0; i < Z.size(); ++i) worst = std::fmax(worst, std::fabs(Z[i] - G[i]));
    CHECK(worst <= 1e-14, "CE dlogits differ from the fused oracle's by %g", worst);
}

// The cut of a launch's last round of tiles along K: whatever the tile count and the K length,
// the cut tiles are the last r <= 16 of every XCD's span, r * s workgroups fit one round of an
// XCD's 32 CUs, every range keeps at least 16 K steps, the ranges partition the K steps, and a
// shorter K never needs more room than a longer one (the plan sizes the room for full chunks).
static void tail_plan_sweep() {
    long cut = 0, all = 0;
    for (int64_t total = 1; total <= 40000; total += (total < 600 ? 1 : 37))
        for (int64_t ksteps = 1; ksteps <= 2100; ksteps += (ksteps < 140 ? 1 : 97)) {
            const flce::TailPlan t = flce::tail_plan(total, ksteps);
            const int64_t per_xcd = (total + 7) / 8;
            ++all;
            CHECK(t.s >= 1 && t.s <= 8, "s out of range");
            CHECK(flce::tail_partial_bytes(total, ksteps) ==
                      (t.s > 1 ? (size_t)8 * t.r * t.s * 256 * 256 * 4 : (size_t)0), "bytes of partial blocks");
            if (ksteps > 1)
                CHECK(flce::tail_partial_bytes(total, ksteps - 1) <= flce::tail_partial_bytes(total, ksteps),
                      "a shorter K needs more room (total %lld ksteps %lld)", (long long)total, (long long)ksteps);
            if (t.s == 1) continue;
            ++cut;
            CHECK(t.r >= 1 && t.r <= 16 && t.r * t.s <= 32, "r %d s %d do not fit a round", t.r, t.s);
            CHECK(t.begin + t.r == per_xcd && t.begin % 32 == 0 && t.begin >= 32, "position of the cut tiles");
            CHECK(ksteps / t.s >= 16, "a range of fewer than 16 K steps");
            int64_t covered = 0, prev_end = 0;
            for (int i = 0; i < t.s; ++i) {
                const int64_t b = ksteps * i / t.s, e = ksteps * (i + 1) / t.s;
                CHECK(b == prev_end && e > b, "K ranges do not tile the K steps");
                covered += e - b;
                prev_end = e;
            }
            CHECK(covered == ksteps, "K steps lost");
        }
    std::printf("tail plan: %ld launches checked, %ld of them cut\n", all, cut);
    CHECK(cut > 0, "no launch was cut");
}

// The deal of a launch's tiles to the XCDs: every tile number below the total comes up exactly
// once over the 8 lists, the tiles from 256 F on are the last ones of every list (where the cut of
// the last round expects them), and a full round is 32 consecutive numbers on one XCD.
static void xcd_deal_sweep() {
    long checked = 0;
    for (int total = 1; total <= 70000; total += (total < 1200 ? 1 : 211)) {
        const int per_xcd = (total + 7) / 8, full = per_xcd / 32 * 32;
        std::vector<unsigned char> seen((size_t)total, 0);
        for (int x = 0; x < 8; ++x)
            for (int i = 0; i < per_xcd; ++i) {
                const int s = flce::xcd_tile_number(x, i, per_xcd);
                CHECK(s >= 0, "negative tile number");
                if (i < full) CHECK(s < 8 * full && s / 32 % 8 == x && s % 32 == i % 32, "round on the wrong XCD");
                else CHECK(s >= 8 * full, "a leftover tile inside the full rounds");
                if (s < total) {
                    CHECK(!seen[(size_t)s], "tile %d dealt twice (total %d)", s, total);
                    seen[(size_t)s] = 1;
                }
                ++checked;
            }
        for (int s = 0; s < total; ++s) CHECK(seen[(size_t)s], "tile %d not dealt (total %d)", s, total);
    }
    std::printf("xcd deal: %ld positions checked\n", checked);
}

static void scheduler_sweep() {
    using flce::Plan;
    const int64_t Hs[] = {1, 8, 64, 100, 512, 2304, 3584, 4096, 8192};
    const int64_t Vs[] = {1, 2, 1000, 4096, 32000, 50257, 128256, 152064, 256000, 1 << 20};
    const int64_t BTs[] = {1, 2, 255, 256, 257, 4096, 8184, 8192, 16384, 131072, 1000003};
    const size_t budgets[] = {1, (size_t)1 << 20, (size_t)1 << 30, (size_t)5 << 29, (size_t)1 << 34};
    long plans = 0;
    for (int dtype = 0; dtype < 2; ++dtype)
        for (int64_t H : Hs)
            for (int64_t V : Vs)
                for (size_t budget : budgets) {
                    const Plan cap = flce::make_plan(0, H, V, dtype, budget, true, true);
                    for (int64_t BT : BTs)
                        for (int compact = 0; compact < 2; ++compact) {
                            const Plan p = flce::make_plan(BT, H, V, dtype, budget, false, compact != 0);
                            ++plans;
                            CHECK(p.nchunks >= 1 && p.C >= 1 && p.nchunks * p.C >= BT, "chunks do not cover BT");
                            CHECK((p.nchunks - 1) * p.C < BT, "an empty chunk");
                            CHECK(p.nchunks == 1 || p.C % flce::CHUNK_ALIGN == 0, "unaligned chunk size");
                            CHECK(p.ldz >= V && p.ldz % 64 == 0 && p.ldc >= p.C, "leading dimensions");
                            const size_t offs[] = {p.off_hdr, p.off_row_loss, p.off_z, p.off_gt, p.off_wt,
                                                   p.off_xt, p.off_dwacc, p.off_dxpart, p.off_xg, p.off_dxg,
                                                   p.off_idx, p.off_tv, p.off_dyn, p.off_tail, p.total};
                            for (size_t k = 0; k + 1 < sizeof(offs) / sizeof(offs[0]); ++k)
                                CHECK(offs[k] % 256 == 0 && offs[k] <= offs[k + 1], "workspace layout");
                            CHECK(p.off_z - p.off_row_loss >= (size_t)p.C * 4, "row losses overlap the logits");
                            CHECK(p.total <= cap.total, "workspace %zu above the bound %zu (BT %lld H %lld V %lld)",
                                  p.total, cap.total, (long long)BT, (long long)H, (long long)V);
                            CHECK(p.dx_ksplit >= 1 && p.dx_ksplit <= 16, "K ranges");
                            CHECK(p.total - p.off_tail >= p.tail_bytes && p.tail_bytes <= ((size_t)64 << 20),
                                  "room for the partial blocks of the dW product's last round");
                        }
                }
    std::printf("scheduler: %ld plans checked\n", plans);
    CHECK(flce::paper_chunk_rows(8192, 4096, 128256) == 256, "paper rule");
}

int main() {
    oracle_case(1, 3, 5, 0, false);      // fewer than four rows
    oracle_case(6, 5, 7, 3, false);      // tail of the four-row sweep, ignored rows
    oracle_case(64, 16, 33, 5, false);   // exactly one row block
    oracle_case(131, 9, 40, 4, false);   // two row blocks and a remainder of three rows
    oracle_case(70, 8, 11, 1, false);    // no valid row at all
    oracle_case(67, 4, 17, 0, true);     // W = 0: loss = log V
    scheduler_sweep();
    tail_plan_sweep();
    xcd_deal_sweep();
    if (failures) {
        std::printf("%d check(s) failed\n", failures);
        return 1;
    }
    std::printf("sanitizer driver: all checks passed\n");
    return 0;
}
