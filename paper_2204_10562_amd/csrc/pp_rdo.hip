// Recursive device ordering (Alg. 2, Sec. IV-B): host code, no kernels.  The ordering is
// computed once per cluster and feeds the batched plan evaluation as one candidate row.
// Every split costs one Stoer-Wagner run, O(n^3) with the dense scans used here, so the
// worst case (a split that peels off one device at a time) is O(D^4): about 15 ms at D = 64
// and 2 s at D = 256 on one host core.
#include <utility>
#include <vector>

#include "pp_common.h"

namespace {

// The graph of one segment while Stoer-Wagner contracts it.  Node i starts as the i-th
// device of the segment; a contracted node keeps the slot of the vertex it was merged into.
struct cut_graph {
    int n;                       // slots (devices of the segment)
    std::vector<int64_t> w;      // n x n symmetric weights between slots
    std::vector<int> lowest;     // lowest device index inside the slot's node
    std::vector<int> slot_of;    // slot of the node that holds the i-th device
    std::vector<char> alive;

    cut_graph(int D, const int64_t *bw, const int32_t *dev, int n_)
        : n(n_), w((size_t)n_ * n_), lowest(n_), slot_of(n_), alive(n_, 1) {
        for (int a = 0; a < n; ++a) {
            lowest[a] = dev[a];
            slot_of[a] = a;
            for (int b = 0; b < n; ++b)
                w[(size_t)a * n + b] =
                    a == b ? 0 : bw[(size_t)dev[a] * D + dev[b]] + bw[(size_t)dev[b] * D + dev[a]];
        }
    }

    // `a` comes before `b` in every tie: the node with the lower lowest device
    bool before(int a, int b) const { return lowest[a] < lowest[b]; }

    // One maximum-adjacency phase.  Returns the weight of the cut that separates the node
    // added last (*last) from all others; *prev is the node added just before it.
    int64_t phase(int live, int *prev, int *last, std::vector<int64_t> &conn,
                  std::vector<char> &taken) const {
        int first = -1;
        for (int a = 0; a < n; ++a)
            if (alive[a] && (first < 0 || before(a, first))) first = a;
        for (int a = 0; a < n; ++a) {
            taken[a] = !alive[a];
            conn[a] = w[(size_t)first * n + a];
        }
        taken[first] = 1;
        int p = first, q = first;
        int64_t cut = 0;
        for (int step = 1; step < live; ++step) {
            int best = -1;
            for (int a = 0; a < n; ++a) {
                if (taken[a]) continue;
                if (best < 0 || conn[a] > conn[best] || (conn[a] == conn[best] && before(a, best)))
                    best = a;
            }
            taken[best] = 1;
            p = q;
            q = best;
            cut = conn[best];
            const int64_t *row = &w[(size_t)best * n];
            for (int a = 0; a < n; ++a) conn[a] += row[a];
        }
        *prev = p;
        *last = q;
        return cut;
    }

    void contract(int into, int from) {
        for (int a = 0; a < n; ++a) {
            int64_t sum = w[(size_t)into * n + a] + w[(size_t)from * n + a];
            w[(size_t)into * n + a] = sum;
            w[(size_t)a * n + into] = sum;
        }
        w[(size_t)into * n + into] = 0;
        if (lowest[from] < lowest[into]) lowest[into] = lowest[from];
        for (int a = 0; a < n; ++a)
            if (slot_of[a] == from) slot_of[a] = into;
        alive[from] = 0;
    }
};

// Minimum cut of the segment dev[0..n-1] (ascending device indices): apart[i] = 1 for the
// devices on the side of the lightest phase cut that was cut OFF (the last-added node).
void lightest_cut(int D, const int64_t *bw, const int32_t *dev, int n, std::vector<char> &apart) {
    cut_graph g(D, bw, dev, n);
    std::vector<int64_t> conn(n);
    std::vector<char> taken(n);
    bool have = false;
    int64_t lightest = 0;
    for (int live = n; live >= 2; --live) {
        int prev, last;
        int64_t cut = g.phase(live, &prev, &last, conn, taken);
        if (!have || cut < lightest) {
            have = true;
            lightest = cut;
            for (int a = 0; a < n; ++a) apart[a] = g.slot_of[a] == last;
        }
        g.contract(prev, last);
    }
}

}  // namespace

extern "C" int pp_rdo_order(int D, const int64_t *bw, int32_t *order_out) {
    if (D < 1 || D > PP_MAX_DEVICES || !bw || !order_out) return PP_ERR_INVALID_ARG;
    // every cut weight is a sum of at most D*D entries: keep it below 2^62
    const int64_t cap = ((int64_t)1 << 62) / ((int64_t)D * D);
    for (int u = 0; u < D; ++u)
        for (int v = 0; v < D; ++v)
            if (u != v && (bw[(size_t)u * D + v] < 0 || bw[(size_t)u * D + v] > cap))
                return PP_ERR_INVALID_ARG;
    for (int i = 0; i < D; ++i) order_out[i] = i;
    // segments [lo, lo+n) of order_out still to be split; each holds ascending devices
    std::vector<std::pair<int, int>> todo;
    todo.emplace_back(0, D);
    std::vector<char> apart;
    std::vector<int32_t> tmp;
    while (!todo.empty()) {
        std::pair<int, int> seg = todo.back();
        todo.pop_back();
        int lo = seg.first, n = seg.second;
        if (n < 2) continue;
        int32_t *dev = order_out + lo;
        apart.assign(n, 0);
        lightest_cut(D, bw, dev, n, apart);
        // the side that holds the segment's lowest device (dev[0]) goes first; both sides
        // keep their ascending order
        char first_side = apart[0];
        tmp.clear();
        for (int i = 0; i < n; ++i)
            if (apart[i] == first_side) tmp.push_back(dev[i]);
        int n1 = (int)tmp.size();
        for (int i = 0; i < n; ++i)
            if (apart[i] != first_side) tmp.push_back(dev[i]);
        for (int i = 0; i < n; ++i) dev[i] = tmp[i];
        todo.emplace_back(lo, n1);
        todo.emplace_back(lo + n1, n - n1);
    }
    return PP_OK;
}
