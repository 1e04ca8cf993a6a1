// Driver for the host-only part of the library under AddressSanitizer and
// UndefinedBehaviorSanitizer: worker divisions, topology patterns and the
// validation/packing of a division, on random valid and invalid inputs.
// Built and run by tests/test_host_sanitizers.py with g++ (no GPU code).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "ds_internal.h"

static uint64_t state = 0x1234567;
static uint64_t next_u64() {
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return state;
}
static int below(int n) { return static_cast<int>(next_u64() % static_cast<uint64_t>(n)); }

int main() {
    long checked = 0;
    // recommended row pitch: extremes first (signed overflow would trip the sanitizer), then random lengths
    const int64_t edge[] = {INT64_MIN, -1, 0, 1, 255, 256, 257, INT64_MAX - 1024, INT64_MAX - 512, INT64_MAX - 511, INT64_MAX};
    for (const int64_t P : edge) {
        const int64_t ld = ds_padded_ld(P);
        if (ld != 0 && (ld < P || ld % 256 != 0 || (ld / 256) % 2 != 1)) { std::printf("ds_padded_ld(%lld) = %lld\n", (long long)P, (long long)ld); return 1; }
    }
    for (int iter = 0; iter < 20000; ++iter) {
        const int64_t P = static_cast<int64_t>(next_u64() >> (1 + below(62)));
        const int64_t ld = ds_padded_ld(P);
        if (ld == 0 ? P <= INT64_MAX - 1024 : (ld < P || ld - P >= 512 || ld % 256 != 0 || (ld / 256) % 2 != 1)) {
            std::printf("ds_padded_ld(%lld) = %lld\n", (long long)P, (long long)ld);
            return 1;
        }
    }
    for (int iter = 0; iter < 20000; ++iter) {
        const int W = 1 + below(DS_MAX_W);
        std::vector<int32_t> sizes;
        int left = W;
        while (left > 0) {
            const int s = 1 + below(left);
            sizes.push_back(s);
            left -= s;
        }
        std::vector<int32_t> perm(static_cast<size_t>(W)), off(sizes.size() + 1);
        int rc = ds_partition(next_u64(), next_u64(), W, sizes.data(), static_cast<int32_t>(sizes.size()), perm.data(),
                              off.data());
        if (rc != DS_OK) { std::printf("ds_partition failed: %d\n", rc); return 1; }
        ds::PartitionArg packed;
        int32_t largest = 0;
        rc = ds::pack_partition(W, perm.data(), off.data(), static_cast<int32_t>(sizes.size()), &packed, &largest);
        if (rc != DS_OK) { std::printf("pack_partition rejected a valid division: %d\n", rc); return 1; }
        // unpack and compare
        for (int q = 0; q < W; ++q) {
            const int got = static_cast<int>((packed.perm[q >> 2] >> ((q & 3) * 8)) & 0xff);
            if (got != perm[static_cast<size_t>(q)]) { std::printf("packing mismatch\n"); return 1; }
        }
        // damaged divisions must be rejected, never read out of bounds
        std::vector<int32_t> bad = perm;
        bad[static_cast<size_t>(below(W))] = below(3) == 0 ? -1 - below(5) : W + below(100);
        if (ds::pack_partition(W, bad.data(), off.data(), static_cast<int32_t>(sizes.size()), &packed, &largest) != DS_ERR_BAD_PART) {
            std::printf("out-of-range worker accepted\n");
            return 1;
        }
        std::vector<int32_t> bad_sizes = sizes;
        bad_sizes[static_cast<size_t>(below(static_cast<int>(sizes.size())))] += 1 + below(3);
        if (ds_partition(1, 2, W, bad_sizes.data(), static_cast<int32_t>(bad_sizes.size()), perm.data(), off.data()) == DS_OK) {
            std::printf("bad sizes accepted\n");
            return 1;
        }

        // topology pattern on a random rack table
        const int R = 1 + below(W < 6 ? W : 6);
        std::vector<int32_t> rack_of(static_cast<size_t>(W));
        for (int w = 0; w < W; ++w) rack_of[static_cast<size_t>(w)] = w < R ? w : below(R);   // every rack used
        std::vector<uint8_t> slow_rack(static_cast<size_t>(R)), slow_worker(static_cast<size_t>(W));
        for (auto& f : slow_rack) f = below(3) == 0;
        for (int w = 0; w < W; ++w) slow_worker[static_cast<size_t>(w)] = w >= R && below(4) == 0;   // rack r keeps worker r free
        std::vector<int32_t> pperm(static_cast<size_t>(W)), poff(static_cast<size_t>(W) + 1);
        int32_t n_groups = 0;
        uint64_t period = 0;
        rc = ds_pattern_period(W, rack_of.data(), slow_rack.data(), R, slow_worker.data(), &period);
        if (rc != DS_OK || period < 1) { std::printf("ds_pattern_period failed: %d\n", rc); return 1; }
        const uint64_t t = next_u64();
        rc = ds_pattern(W, rack_of.data(), slow_rack.data(), R, slow_worker.data(), t, pperm.data(), poff.data(), &n_groups);
        if (rc != DS_OK) { std::printf("ds_pattern failed: %d\n", rc); return 1; }
        rc = ds::pack_partition(W, pperm.data(), poff.data(), n_groups, &packed, &largest);
        if (rc != DS_OK) { std::printf("pattern is not a valid division: %d\n", rc); return 1; }
        std::vector<int32_t> again(static_cast<size_t>(W)), again_off(static_cast<size_t>(W) + 1);
        int32_t n_again = 0;
        rc = ds_pattern(W, rack_of.data(), slow_rack.data(), R, slow_worker.data(), t + period, again.data(), again_off.data(), &n_again);
        if (rc != DS_OK || n_again != n_groups || again != pperm) { std::printf("pattern is not periodic\n"); return 1; }
        // premise of the consensus bound on one period of the pattern (capped) and on a damaged list;
        // every 50th round only: the fp64 matrix powers are slow under the sanitizers
        if (iter % 50 == 0) {
            const int Bp = static_cast<int>(period < 24 ? period : 24);
            std::vector<int32_t> perms(static_cast<size_t>(Bp) * W), offs(static_cast<size_t>(Bp) * (W + 1)), counts(static_cast<size_t>(Bp));
            for (int k = 0; k < Bp; ++k) {
                rc = ds_pattern(W, rack_of.data(), slow_rack.data(), R, slow_worker.data(), t + static_cast<uint64_t>(k),
                                perms.data() + static_cast<size_t>(k) * W, offs.data() + static_cast<size_t>(k) * (W + 1),
                                &counts[static_cast<size_t>(k)]);
                if (rc != DS_OK) { std::printf("ds_pattern failed inside a period: %d\n", rc); return 1; }
            }
            int32_t connected = -1;
            double rho = -1.0, sigma = -1.0;
            rc = ds_pattern_check(W, Bp, perms.data(), offs.data(), counts.data(), &connected, &rho, &sigma);
            if (rc != DS_OK || connected < 0 || !(rho >= 0.0 && rho <= 1.0 + 1e-9) || !(sigma >= rho - 1e-9 && sigma <= 1.0 + 1e-9) ||
                (connected == 1) != (sigma < 1.0 - 1e-9)) {
                std::printf("ds_pattern_check: rc %d connected %d rho %g sigma %g\n", rc, connected, rho, sigma);
                return 1;
            }
            // (a full period need not be connected: a rack whose only worker without NIC contention is
            //  always its representative never mixes its other workers with anybody else)
            perms[static_cast<size_t>(below(Bp * W))] = W + below(50);
            if (ds_pattern_check(W, Bp, perms.data(), offs.data(), counts.data(), &connected, &rho, &sigma) != DS_ERR_BAD_PART) {
                std::printf("ds_pattern_check accepted a damaged list\n");
                return 1;
            }
        }
        rack_of[static_cast<size_t>(below(W))] = R + below(4);   // rack index out of range
        if (ds_pattern(W, rack_of.data(), slow_rack.data(), R, slow_worker.data(), t, pperm.data(), poff.data(), &n_groups) != DS_ERR_TOPOLOGY) {
            std::printf("bad rack index accepted\n");
            return 1;
        }
        ++checked;
    }
    std::printf("ok %ld\n", checked);
    return 0;
}
