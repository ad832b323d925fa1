// Host-only driver for sanitizer runs: exercises argument validation and the
// launch-plan builder (odsgd_plan_host, odsgd_workspace_bytes, odsgd_strerror)
// over many shapes, alignments and error cases.  No device call is made.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "odsgd.h"

static uint64_t rng_state = 88172645463325252ull;
static uint64_t rnd() { rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17; return rng_state; }

int main()
{
    int plans = 0, rejected = 0;
    for (int iter = 0; iter < 400; ++iter) {
        const int K = 1 + (int)(rnd() % 6), W = 1 + (int)(rnd() % 9);
        std::vector<int64_t> numel(K);
        for (auto &n : numel) { uint64_t r = rnd() % 5; n = r == 0 ? (int64_t)(rnd() % 5) : r == 1 ? (int64_t)(rnd() % 700) : r == 2 ? (int64_t)(rnd() % 70000) : (int64_t)(rnd() % 20000); }
        const int roles = 2 + 2 * W;
        std::vector<std::vector<float *>> ptr(roles, std::vector<float *>(K));
        const unsigned kind = (unsigned)(rnd() % 5);
        for (int j = 0; j < roles; ++j) {
            uintptr_t a = 0x7f0000000000ull + (uintptr_t)j * (1ull << 36);
            const uintptr_t phase = kind == 0 ? 0 : kind == 1 ? 16 * (1 + iter % 60) : kind == 2 ? 4 * (1 + iter % 250)
                                    : kind == 3 ? 16 * (rnd() % 64) : 4 * (rnd() % 256);
            // kinds 0-2: every role has the same offset from a 64 KiB boundary (two-half tiles possible)
            for (int k = 0; k < K; ++k) { ptr[j][k] = (float *)(a + phase); a += ((4 * (uintptr_t)numel[k] + phase + 65535) / 65536 + 1) * 65536; }
        }
        if (iter % 17 == 3) ptr[2 + W][0] = ptr[0][0];           // local weights alias w
        if (iter % 23 == 5) ptr[1][K - 1] = (float *)((uintptr_t)ptr[1][K - 1] + 2);  // misaligned
        std::vector<const float *const *> grads(W);
        std::vector<float *const *> locals(W);
        std::vector<std::vector<const float *>> gconst(W, std::vector<const float *>(K));
        for (int m = 0; m < W; ++m) {
            for (int k = 0; k < K; ++k) gconst[m][k] = ptr[2 + m][k];
            grads[m] = gconst[m].data();
            locals[m] = ptr[2 + W + m].data();
        }
        const size_t bytes = odsgd_workspace_bytes(K, numel.data(), W);
        if (bytes == 0) { std::printf("workspace query failed\n"); return 1; }
        std::vector<unsigned char> image(bytes);
        int64_t nrows = -1, nchunks = -1; size_t off = 0;
        const int rc = odsgd_plan_host(K, numel.data(), ptr[0].data(), ptr[1].data(), grads.data(), locals.data(), W,
                                       image.data(), image.size(), &nrows, &nchunks, &off);
        if (rc != ODSGD_OK) { ++rejected; (void)odsgd_strerror(rc); continue; }
        ++plans;
        // every element covered exactly once
        std::vector<std::vector<unsigned char>> seen(K);
        for (int k = 0; k < K; ++k) seen[k].assign((size_t)numel[k], 0);
        const uint32_t *ct = (const uint32_t *)(image.data() + off);
        if (nrows != K) { std::printf("one row per tensor expected\n"); return 1; }
        for (int64_t c = 0; c < nchunks; ++c) {
            const uint32_t t = ct[4 * c] & 0x7fffffffu, cnt = ct[4 * c + 1], o = ct[4 * c + 2], second = ct[4 * c + 3];
            if ((int)t >= K) { std::printf("chunk row out of range\n"); return 1; }
            for (uint32_t i = 0; i < cnt; ++i) {
                // a two-half tile: lanes 32..63 (elements 128..255) sit 4 * second elements further on
                const uint64_t e = (uint64_t)o + i + ((second && i >= 128) ? 4ull * second : 0ull);
                if (e >= (uint64_t)numel[t]) { std::printf("chunk out of range\n"); return 1; }
                if (seen[t][e]++) { std::printf("element covered twice\n"); return 1; }
            }
        }
        for (int k = 0; k < K; ++k) for (auto s : seen[k]) if (!s) { std::printf("element not covered\n"); return 1; }
        // too-small image is refused, not overrun
        if (odsgd_plan_host(K, numel.data(), ptr[0].data(), ptr[1].data(), grads.data(), locals.data(), W,
                            image.data(), 8, &nrows, &nchunks, &off) != ODSGD_ENOSPC) { std::printf("ENOSPC expected\n"); return 1; }
    }
    if (odsgd_workspace_bytes(0, nullptr, 1) != 0 || odsgd_step(nullptr, nullptr, nullptr) != ODSGD_EINVAL) return 1;
    std::printf("ok plans=%d rejected=%d\n", plans, rejected);
    return plans > 100 && rejected > 10 ? 0 : 1;
}
