// Topology-aware divide-and-shuffle pattern (Sec. III-B: static topology
// heterogeneity, inter-rack link contention, end-host NIC contention).
// Host-only integer code: the division of iteration t is computed directly
// from t (nothing is carried between iterations), so it can stand in for
// ds_partition wherever the rack of every worker is known.
#include <cmath>
#include <numeric>

#include "ds_internal.h"

namespace {

struct Topology {
    int32_t n_racks = 0;
    int32_t n_members[DS_MAX_W] = {};            // workers per rack
    int32_t members[DS_MAX_W][DS_MAX_W] = {};    // ascending worker index
    int32_t n_free[DS_MAX_W] = {};               // workers without NIC contention per rack
    int32_t free_members[DS_MAX_W][DS_MAX_W] = {};
};

int read_topology(int32_t W, const int32_t* rack_of, const uint8_t* slow_rack, int32_t n_racks,
                  const uint8_t* slow_worker, Topology* topo) {
    if (!rack_of || !slow_rack || !slow_worker) return DS_ERR_NULL;
    if (W < 1 || W > DS_MAX_W) return DS_ERR_BAD_W;
    if (n_racks < 1 || n_racks > W) return DS_ERR_TOPOLOGY;
    topo->n_racks = n_racks;
    for (int32_t w = 0; w < W; ++w) {
        const int32_t r = rack_of[w];
        if (r < 0 || r >= n_racks) return DS_ERR_TOPOLOGY;
        topo->members[r][topo->n_members[r]++] = w;
        if (!slow_worker[w]) topo->free_members[r][topo->n_free[r]++] = w;
    }
    for (int32_t r = 0; r < n_racks; ++r) {
        if (topo->n_members[r] == 0) return DS_ERR_TOPOLOGY;   // rack indices must be dense
        if (topo->n_free[r] == 0) return DS_ERR_TOPOLOGY;      // someone must be able to represent the rack
    }
    return DS_OK;
}

struct Writer {
    int32_t* perm;
    int32_t* off;
    int32_t n_workers = 0;
    int32_t n_groups = 0;
    void add(int32_t w) { perm[n_workers++] = w; }
    void close_group() { off[++n_groups] = n_workers; }
};

}  // namespace

extern "C" int ds_pattern(int32_t W, const int32_t* rack_of, const uint8_t* slow_rack, int32_t n_racks,
                          const uint8_t* slow_worker, uint64_t t, int32_t* perm_out, int32_t* off_out,
                          int32_t* n_groups_out) {
    if (!perm_out || !off_out || !n_groups_out) return DS_ERR_NULL;
    Topology topo;
    const int rc = read_topology(W, rack_of, slow_rack, n_racks, slow_worker, &topo);
    if (rc != DS_OK) return rc;

    Writer out{perm_out, off_out};
    off_out[0] = 0;
    int32_t rep[DS_MAX_W];
    const bool has_links = n_racks >= 2;
    for (int32_t r = 0; r < n_racks; ++r)
        rep[r] = has_links ? topo.free_members[r][t % static_cast<uint64_t>(topo.n_free[r])] : -1;

    if (has_links) {
        int32_t delayed[DS_MAX_W], regular[DS_MAX_W], n_delayed = 0, n_regular = 0;
        for (int32_t r = 0; r < n_racks; ++r) (slow_rack[r] ? delayed[n_delayed++] : regular[n_regular++]) = r;
        if (n_delayed == 0 || n_regular == 0) {
            for (int32_t r = 0; r < n_racks; ++r) out.add(rep[r]);
            out.close_group();
        } else {
            // each delayed representative gets one regular partner, a different one every iteration
            bool taken[DS_MAX_W] = {};
            const int32_t n_pairs = n_delayed < n_regular ? n_delayed : n_regular;
            for (int32_t k = 0; k < n_pairs; ++k) {
                const int32_t partner = regular[(t + static_cast<uint64_t>(k)) % static_cast<uint64_t>(n_regular)];
                taken[partner] = true;
                out.add(rep[delayed[k]]);
                out.add(rep[partner]);
                out.close_group();
            }
            for (int32_t k = n_pairs; k < n_delayed; k += 2) {   // more delayed than regular racks
                out.add(rep[delayed[k]]);
                if (k + 1 < n_delayed) out.add(rep[delayed[k + 1]]);
                out.close_group();
            }
            bool any = false;
            for (int32_t i = 0; i < n_regular; ++i) {
                if (!taken[regular[i]]) {
                    out.add(rep[regular[i]]);
                    any = true;
                }
            }
            if (any) out.close_group();
        }
    }

    for (int32_t r = 0; r < n_racks; ++r) {
        int32_t slow[DS_MAX_W], fast[DS_MAX_W], n_slow = 0, n_fast = 0;
        for (int32_t i = 0; i < topo.n_members[r]; ++i) {
            const int32_t w = topo.members[r][i];
            if (w == rep[r]) continue;
            (slow_worker[w] ? slow[n_slow++] : fast[n_fast++]) = w;
        }
        if (n_slow > 0 && n_fast > n_slow) {
            // every delayed worker is paired with a regular one; the rest is the rack's hub
            bool used[DS_MAX_W] = {};
            for (int32_t k = 0; k < n_slow; ++k) {
                const int32_t pick = static_cast<int32_t>((t + static_cast<uint64_t>(k)) % static_cast<uint64_t>(n_fast));
                used[pick] = true;
                out.add(slow[k]);
                out.add(fast[pick]);
                out.close_group();
            }
            for (int32_t i = 0; i < n_fast; ++i)
                if (!used[i]) out.add(fast[i]);
            out.close_group();
        } else if (n_slow + n_fast > 0) {
            // not split: the order is that of the rack (ascending worker index)
            for (int32_t i = 0; i < topo.n_members[r]; ++i)
                if (topo.members[r][i] != rep[r]) out.add(topo.members[r][i]);
            out.close_group();
        }
    }
    *n_groups_out = out.n_groups;
    return DS_OK;
}

extern "C" int ds_pattern_period(int32_t W, const int32_t* rack_of, const uint8_t* slow_rack, int32_t n_racks,
                                 const uint8_t* slow_worker, uint64_t* period_out) {
    if (!period_out) return DS_ERR_NULL;
    Topology topo;
    const int rc = read_topology(W, rack_of, slow_rack, n_racks, slow_worker, &topo);
    if (rc != DS_OK) return rc;
    uint64_t period = 1;
    auto fold = [&period](int64_t n) {
        if (n > 0) period = std::lcm(period, static_cast<uint64_t>(n));
    };
    const bool has_links = n_racks >= 2;
    int32_t n_regular = 0;
    for (int32_t r = 0; r < n_racks; ++r) {
        if (!slow_rack[r]) ++n_regular;
        if (has_links) fold(topo.n_free[r]);                       // turns as representative
        const int32_t n_slow = topo.n_members[r] - topo.n_free[r];
        const int32_t n_fast_inside = topo.n_free[r] - (has_links ? 1 : 0);
        if (n_slow > 0 && n_fast_inside > n_slow) fold(n_fast_inside);   // partner of the small intra-rack group
    }
    if (has_links && n_regular > 0 && n_regular < n_racks) fold(n_regular);   // partner of the delayed racks
    *period_out = period;
    return DS_OK;
}

// ---------------------------------------------------------------- premise of the consensus bound

namespace {

constexpr int kN = DS_MAX_W;
typedef double Matrix[kN][kN];   // the leading n x n block is used

double frobenius(const Matrix& a, int n) {
    double s = 0.0;
    for (int i = 0; i < n; ++i)
        for (int j = 0; j < n; ++j) s += a[i][j] * a[i][j];
    return std::sqrt(s);
}

// Spectral radius of a (destroyed) by Gelfand's formula along the powers 2^j:
// with a_0 = a and a_{j+1} = (a_j / ||a_j||)^2,  log rho = sum_j log||a_j|| / 2^j.
// Every factor is normalised before it is squared, so nothing over- or
// underflows, and after 64 squarings the neglected tail weighs 2^-64.
double spectral_radius(Matrix& a, Matrix& tmp, int n) {
    double log_rho = 0.0, weight = 1.0;
    for (int iter = 0; iter < 64; ++iter) {
        const double norm = frobenius(a, n);
        if (!(norm > 0.0)) return 0.0;   // nilpotent: every eigenvalue is 0
        log_rho += weight * std::log(norm);
        weight *= 0.5;
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) tmp[i][j] = a[i][j] / norm;
        for (int i = 0; i < n; ++i) {
            for (int j = 0; j < n; ++j) {
                double s = 0.0;
                for (int k = 0; k < n; ++k) s += tmp[i][k] * tmp[k][j];
                a[i][j] = s;
            }
        }
    }
    return std::exp(log_rho);
}

int find_root(int32_t* parent, int v) {
    while (parent[v] != v) {
        parent[v] = parent[parent[v]];
        v = parent[v];
    }
    return v;
}

}  // namespace

extern "C" int ds_pattern_check(int32_t W, int32_t B, const int32_t* perms, const int32_t* offs,
                                const int32_t* n_groups, int32_t* connected_out, double* rho_out,
                                double* sigma_out) {
    if (!perms || !offs || !n_groups || !connected_out) return DS_ERR_NULL;
    if (W < 1 || W > DS_MAX_W) return DS_ERR_BAD_W;
    if (B < 1) return DS_ERR_BAD_SHAPE;
    ds::PartitionArg unused;
    int32_t largest = 0;
    for (int32_t k = 0; k < B; ++k) {
        const int rc = ds::pack_partition(W, perms + static_cast<int64_t>(k) * W, offs + static_cast<int64_t>(k) * (W + 1),
                                          n_groups[k], &unused, &largest);
        if (rc != DS_OK) return rc;
    }

    // connectivity of the union of the groups over the period
    int32_t parent[DS_MAX_W];
    for (int32_t w = 0; w < W; ++w) parent[w] = w;
    for (int32_t k = 0; k < B; ++k) {
        const int32_t* perm = perms + static_cast<int64_t>(k) * W;
        const int32_t* off = offs + static_cast<int64_t>(k) * (W + 1);
        for (int32_t g = 0; g < n_groups[k]; ++g)
            for (int32_t q = off[g] + 1; q < off[g + 1]; ++q)
                parent[find_root(parent, perm[q])] = find_root(parent, perm[off[g]]);
    }
    int32_t components = 0;
    for (int32_t w = 0; w < W; ++w) components += find_root(parent, w) == w;
    *connected_out = components == 1;
    if (!rho_out && !sigma_out) return DS_OK;

    // M = W_{B-1} ... W_0: applying W_k on the left replaces the rows of a group by their mean
    Matrix m, a, tmp;   // 3 x 32 KiB on the stack
    for (int i = 0; i < W; ++i)
        for (int j = 0; j < W; ++j) m[i][j] = i == j ? 1.0 : 0.0;
    for (int32_t k = 0; k < B; ++k) {
        const int32_t* perm = perms + static_cast<int64_t>(k) * W;
        const int32_t* off = offs + static_cast<int64_t>(k) * (W + 1);
        for (int32_t g = 0; g < n_groups[k]; ++g) {
            const int32_t n = off[g + 1] - off[g];
            if (n == 1) continue;
            for (int j = 0; j < W; ++j) {
                double s = 0.0;
                for (int32_t q = off[g]; q < off[g + 1]; ++q) s += m[perm[q]][j];
                s /= static_cast<double>(n);
                for (int32_t q = off[g]; q < off[g + 1]; ++q) m[perm[q]][j] = s;
            }
        }
    }
    // the part of M that acts on what is orthogonal to consensus
    const double mean = 1.0 / static_cast<double>(W);
    for (int i = 0; i < W; ++i)
        for (int j = 0; j < W; ++j) m[i][j] -= mean;
    if (rho_out) {
        for (int i = 0; i < W; ++i)
            for (int j = 0; j < W; ++j) a[i][j] = m[i][j];
        *rho_out = spectral_radius(a, tmp, W);
    }
    if (sigma_out) {
        for (int i = 0; i < W; ++i) {
            for (int j = 0; j < W; ++j) {
                double s = 0.0;
                for (int k = 0; k < W; ++k) s += m[k][i] * m[k][j];
                a[i][j] = s;
            }
        }
        *sigma_out = std::sqrt(spectral_radius(a, tmp, W));
    }
    return DS_OK;
}
