// Partition loading order and bucket iteration order (paper Sec. 4, Alg. 1 and Alg. 2).
// Host-only.  Buffer capacity is three; one partition is swapped per buffer state; the
// partition swapped in is never the next one swapped out (Theorem 1, property (1)),
// so each swap can overlap the buckets that do not involve the partition being evicted.
#include <cstdint>
#include <cstring>
#include <new>
#include <vector>

#include "legend.h"

namespace {

struct Cover {
    int n;
    std::vector<uint8_t> bit;
    explicit Cover(int n_) : n(n_), bit((size_t)n_ * n_, 0) {}
    bool get(int a, int b) const { return bit[(size_t)a * n + b] != 0; }
    void mark3(const int buf[3]) {
        for (int x = 0; x < 3; ++x)
            for (int y = 0; y < 3; ++y)
                if (buf[x] >= 0 && buf[y] >= 0) bit[(size_t)buf[x] * n + buf[y]] = 1;
    }
    bool row_full(int r) const {
        for (int b = 0; b < n; ++b)
            if (!get(r, b)) return false;
        return true;
    }
    bool all() const {
        for (uint8_t v : bit)
            if (!v) return false;
        return true;
    }
};

int slot_of(const int buf[3], int p) {
    for (int s = 0; s < 3; ++s)
        if (buf[s] == p) return s;
    return -1;
}

// Alg. 1: column-separation covering.  States keep residents in their buffer slot.
std::vector<int> build_states(int n) {
    std::vector<int> st;
    auto push = [&](const int b[3]) { st.insert(st.end(), b, b + 3); };
    if (n <= 3) {
        int b[3] = {-1, -1, -1};
        for (int p = 0; p < n; ++p) b[p] = p;
        push(b);
        return st;
    }
    Cover cov(n);
    int buf[3] = {0, 1, 2};
    push(buf);
    cov.mark3(buf);
    // column 0: bring in 3 .. n-1 in id order, each replacing the partition loaded two states before
    for (int p = 3; p < n; ++p) {
        buf[slot_of(buf, p - 2)] = p;
        push(buf);
        cov.mark3(buf);
    }
    int col = 0;
    int newest = n - 1;
    while (!cov.all()) {
        int evict;
        if (cov.row_full(col)) {
            const int next_col = col + 1;
            if (slot_of(buf, next_col) >= 0) {      // successor already resident: the column just advances
                col = next_col;
                continue;
            }
            buf[slot_of(buf, col)] = next_col;
            push(buf);
            cov.mark3(buf);
            col = next_col;
            newest = next_col;
            if (cov.all()) break;
            int lo = -1, hi = -1;
            for (int s = 0; s < 3; ++s) {
                if (buf[s] == col) continue;
                if (lo < 0 || buf[s] < lo) lo = buf[s];
                if (buf[s] > hi) hi = buf[s];
            }
            bool open_beyond = false;
            for (int x = hi + 1; x < n; ++x)
                if (!cov.get(col, x)) open_beyond = true;
            evict = open_beyond ? hi : lo;
        } else {
            evict = -1;
            for (int s = 0; s < 3; ++s)
                if (buf[s] != col && buf[s] != newest) evict = buf[s];
        }
        int stay[2], ns = 0, top = -1;
        for (int s = 0; s < 3; ++s) {
            if (buf[s] != evict) stay[ns++] = buf[s];
            if (buf[s] > top) top = buf[s];
        }
        int best = -1, best_gain = -1;
        for (int t = 0; t < n; ++t) {
            const int cand = (top + 1 + t) % n;
            if (slot_of(buf, cand) >= 0) continue;
            int gain = 0;
            for (int k = 0; k < ns; ++k)
                if (!cov.get(stay[k], cand)) ++gain;
            if (gain > best_gain) { best = cand; best_gain = gain; }
        }
        buf[slot_of(buf, evict)] = best;
        newest = best;
        push(buf);
        cov.mark3(buf);
    }
    return st;
}

}  // namespace

static int plan_order(int32_t n, int32_t* states, int32_t state_capacity, int32_t* num_states,
                      int32_t* buckets, int32_t* state_begin, int32_t* state_overlap) {
    if (n < 1 || !states || !num_states || !buckets || !state_begin || !state_overlap) return LEGEND_E_INVAL;
    const std::vector<int> st = build_states(n);
    const int ns = (int)(st.size() / 3);
    *num_states = ns;
    if (ns > state_capacity) return LEGEND_E_INVAL;
    for (size_t k = 0; k < st.size(); ++k) states[k] = st[k];

    // Alg. 2: in each state, the untrained buckets that involve the partition evicted next come
    // first (those pairing it with the partition loaded last at the end of that group); the
    // others can run while the swap is in flight.  The last state trains whatever is left.
    std::vector<uint8_t> done((size_t)n * n, 0);
    int nbk = 0;
    auto take = [&](int a, int b) {
        if (!done[(size_t)a * n + b]) {
            done[(size_t)a * n + b] = 1;
            buckets[2 * nbk] = a;
            buckets[2 * nbk + 1] = b;
            ++nbk;
        }
    };
    int newest = -1;
    for (int k = 0; k < ns; ++k) {
        const int* cur = &st[3 * k];
        int evict = -1, load = -1;
        if (k + 1 < ns) {
            const int* nx = &st[3 * (k + 1)];
            for (int s = 0; s < 3; ++s)
                if (cur[s] != nx[s]) { evict = cur[s]; load = nx[s]; }
        }
        state_begin[k] = nbk;
        if (evict >= 0) {
            for (int pass = 0; pass < 2; ++pass)
                for (int s = 0; s < 3; ++s) {
                    const int p = cur[s];
                    if (p < 0 || (pass == 0) == (p == newest)) continue;
                    take(evict, p);
                    take(p, evict);
                }
        }
        state_overlap[k] = nbk;
        int sorted[3] = {cur[0], cur[1], cur[2]};
        for (int a = 0; a < 3; ++a)
            for (int b = a + 1; b < 3; ++b)
                if (sorted[b] < sorted[a]) { int t = sorted[a]; sorted[a] = sorted[b]; sorted[b] = t; }
        for (int a = 0; a < 3; ++a)
            for (int b = 0; b < 3; ++b)
                if (sorted[a] >= 0 && sorted[b] >= 0 && sorted[a] != evict && sorted[b] != evict) take(sorted[a], sorted[b]);
        newest = load;
    }
    state_begin[ns] = nbk;
    return nbk == n * n ? LEGEND_OK : LEGEND_E_STATE;
}

// no C++ exception (the planner's containers can throw std::bad_alloc) crosses the C ABI
extern "C" int legend_plan_order(int32_t n, int32_t* states, int32_t state_capacity, int32_t* num_states,
                                 int32_t* buckets, int32_t* state_begin, int32_t* state_overlap) {
    try {
        return plan_order(n, states, state_capacity, num_states, buckets, state_begin, state_overlap);
    } catch (const std::bad_alloc&) {
        return LEGEND_E_NOMEM;
    } catch (...) {
        return LEGEND_E_STATE;
    }
}
