// Calls the C-ABI of libcolbandit.so from a plain C++ host program: no Python, no torch.
// Device memory comes from hipMalloc, the stream from hipStreamCreate; every scoring step
// runs in the library.  The program checks
//   - colbandit_full_maxsim (fp32 inputs) against the definition (paper Eq. (1)-(2)) written
//     as three loops in double precision, relative tolerance 1e-5, and its top-K against a
//     full sort (Eq. (3));
//   - colbandit_topk: every returned score equals the exhaustive path's score of that
//     document bit for bit (Sec. 4.2, exact rescore), ids are distinct and valid, the
//     accounting identity cells_rescore = T * |A_final| holds;
//   - colbandit_doc_uniform with every cell revealed returns the exhaustive ranking.
// Test infrastructure: built by build.py next to this file and run by the GPU test suite.
// Exit status 0 = all checks passed; a message names the first failure otherwise.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/colbandit.h"

#define HIPOK(x)                                                                         \
    do {                                                                                 \
        hipError_t e_ = (x);                                                             \
        if (e_ != hipSuccess) {                                                          \
            std::fprintf(stderr, "abi_check: %s -> %s\n", #x, hipGetErrorString(e_));   \
            return 2;                                                                    \
        }                                                                                \
    } while (0)
#define CBOK(x)                                                                          \
    do {                                                                                 \
        int r_ = (x);                                                                    \
        if (r_ != COLBANDIT_OK) {                                                        \
            std::fprintf(stderr, "abi_check: %s -> %s\n", #x, colbandit_strerror(r_));  \
            return 3;                                                                    \
        }                                                                                \
    } while (0)
#define CHECK(c)                                                                         \
    do {                                                                                 \
        if (!(c)) {                                                                      \
            std::fprintf(stderr, "abi_check: check failed at line %d: %s\n", __LINE__, #c); \
            return 1;                                                                    \
        }                                                                                \
    } while (0)

static uint64_t lcg_state = 0x2545F4914F6CDD1Dull;
static double unit_rand() {   // in (-1, 1)
    lcg_state = lcg_state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(lcg_state >> 11) / 9007199254740992.0 * 2.0 - 1.0;
}
static void unit_rows(std::vector<float>& x, size_t rows, int d) {
    for (size_t r = 0; r < rows; ++r) {
        double s = 0.0;
        for (int k = 0; k < d; ++k) {
            x[r * d + k] = (float)unit_rand();
            s += (double)x[r * d + k] * x[r * d + k];
        }
        for (int k = 0; k < d; ++k) x[r * d + k] = (float)(x[r * d + k] / std::sqrt(s));
    }
}

int main() {
    const int nq = 2, T = 32, d = 128, K = 5, M = 5;
    const int64_t N = 300;
    std::vector<int64_t> off(N + 1, 0);
    for (int64_t i = 0; i < N; ++i) {
        lcg_state = lcg_state * 6364136223846793005ull + 1442695040888963407ull;
        off[i + 1] = off[i] + 1 + (int64_t)((lcg_state >> 33) % 70);
    }
    const int64_t total = off[N];
    std::vector<float> Q((size_t)nq * T * d), E((size_t)total * d);
    unit_rows(Q, (size_t)nq * T, d);
    unit_rows(E, (size_t)total, d);

    HIPOK(hipSetDevice(0));
    hipStream_t st;
    HIPOK(hipStreamCreate(&st));
    float *dQ, *dE, *dS, *dTopS, *dCbS, *dUS;
    int64_t *dOff, *dTopI, *dCbI, *dUI;
    void* ws;
    const size_t wsb = std::max(colbandit_workspace_bytes(nq, T, d, N, total, K, M),
                                colbandit_doc_uniform_workspace_bytes(nq, T, d, N, total));
    CHECK(wsb > 0);
    HIPOK(hipMalloc(&dQ, Q.size() * 4));
    HIPOK(hipMalloc(&dE, E.size() * 4));
    HIPOK(hipMalloc(&dOff, off.size() * 8));
    HIPOK(hipMalloc(&dS, (size_t)nq * N * 4));
    HIPOK(hipMalloc(&dTopI, (size_t)nq * K * 8));
    HIPOK(hipMalloc(&dTopS, (size_t)nq * K * 4));
    HIPOK(hipMalloc(&dCbI, (size_t)nq * K * 8));
    HIPOK(hipMalloc(&dCbS, (size_t)nq * K * 4));
    HIPOK(hipMalloc(&dUI, (size_t)nq * K * 8));
    HIPOK(hipMalloc(&dUS, (size_t)nq * K * 4));
    HIPOK(hipMalloc(&ws, wsb));
    HIPOK(hipMemcpyAsync(dQ, Q.data(), Q.size() * 4, hipMemcpyHostToDevice, st));
    HIPOK(hipMemcpyAsync(dE, E.data(), E.size() * 4, hipMemcpyHostToDevice, st));
    HIPOK(hipMemcpyAsync(dOff, off.data(), off.size() * 8, hipMemcpyHostToDevice, st));

    CBOK(colbandit_validate_offsets(dOff, N, total, ws, wsb, st));
    CBOK(colbandit_full_maxsim(dQ, nq, T, d, COLBANDIT_F32, dE, dOff, N, total, K, dS, dTopI, dTopS,
                               nullptr, nullptr, ws, wsb, st));
    std::vector<colbandit_stats> stats(nq);
    CBOK(colbandit_topk(dQ, nq, T, d, COLBANDIT_F32, dE, dOff, N, total, K, 0.2f, 0.01f, M, 7ull,
                        nullptr, dCbI, dCbS, stats.data(), ws, wsb, st));
    CBOK(colbandit_doc_uniform(dQ, nq, T, d, COLBANDIT_F32, dE, dOff, N, total, K, T, 11ull, nullptr,
                               nullptr, dUI, dUS, ws, wsb, st));

    std::vector<float> S((size_t)nq * N), topS(nq * K), cbS(nq * K);
    std::vector<int64_t> topI(nq * K), cbI(nq * K), uI(nq * K);
    HIPOK(hipMemcpyAsync(S.data(), dS, S.size() * 4, hipMemcpyDeviceToHost, st));
    HIPOK(hipMemcpyAsync(topS.data(), dTopS, topS.size() * 4, hipMemcpyDeviceToHost, st));
    HIPOK(hipMemcpyAsync(topI.data(), dTopI, topI.size() * 8, hipMemcpyDeviceToHost, st));
    HIPOK(hipMemcpyAsync(cbS.data(), dCbS, cbS.size() * 4, hipMemcpyDeviceToHost, st));
    HIPOK(hipMemcpyAsync(cbI.data(), dCbI, cbI.size() * 8, hipMemcpyDeviceToHost, st));
    HIPOK(hipMemcpyAsync(uI.data(), dUI, uI.size() * 8, hipMemcpyDeviceToHost, st));
    HIPOK(hipStreamSynchronize(st));

    for (int q = 0; q < nq; ++q) {
        // the definition, in double
        std::vector<double> want(N);
        for (int64_t i = 0; i < N; ++i) {
            double s = 0.0;
            for (int t = 0; t < T; ++t) {
                double best = -INFINITY;
                for (int64_t j = off[i]; j < off[i + 1]; ++j) {
                    double dot = 0.0;
                    for (int k = 0; k < d; ++k)
                        dot += (double)Q[((size_t)q * T + t) * d + k] * (double)E[(size_t)j * d + k];
                    best = std::max(best, dot);
                }
                s += best;
            }
            want[i] = s;
            CHECK(std::fabs((double)S[(size_t)q * N + i] - s) <= 1e-5 * std::max(1.0, std::fabs(s)));
        }
        // top-K of the library's own scores: (score descending, index ascending)
        std::vector<int64_t> order(N);
        for (int64_t i = 0; i < N; ++i) order[i] = i;
        const float* Sq = &S[(size_t)q * N];
        std::sort(order.begin(), order.end(),
                  [&](int64_t a, int64_t b) { return Sq[a] != Sq[b] ? Sq[a] > Sq[b] : a < b; });
        for (int k = 0; k < K; ++k) {
            CHECK(topI[q * K + k] == order[k]);
            CHECK(topS[q * K + k] == Sq[order[k]]);
            CHECK(uI[q * K + k] == order[k]);              // Doc-Uniform with every cell revealed
        }
        // Col-Bandit: exact scores of valid, distinct documents
        for (int k = 0; k < K; ++k) {
            const int64_t id = cbI[q * K + k];
            CHECK(id >= 0 && id < N);
            CHECK(cbS[q * K + k] == Sq[id]);
            for (int k2 = 0; k2 < k; ++k2) CHECK(cbI[q * K + k2] != id);
        }
        const colbandit_stats& s = stats[q];
        CHECK(s.rounds >= 1 && s.rounds <= (T + 3) / 4);
        CHECK(s.survivors[0] == N && s.survivors[s.rounds] >= K);
        CHECK(s.cells_rescore == (int64_t)T * s.survivors[s.rounds]);
    }
    void* bufs[] = {dQ, dE, dOff, dS, dTopI, dTopS, dCbI, dCbS, dUI, dUS, ws};
    for (void* p : bufs) HIPOK(hipFree(p));
    HIPOK(hipStreamDestroy(st));
    std::printf("abi_check ok: N=%lld tokens=%lld nq=%d rounds=[%d,%d]\n", (long long)N,
                (long long)total, nq, stats[0].rounds, stats[1].rounds);
    return 0;
}
