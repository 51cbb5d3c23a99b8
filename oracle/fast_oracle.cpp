// CPU oracle for FAST All-to-All(v) schedule synthesis.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded, obviously
// correct statement of what the synthesis path computes.  It exists so that the
// tests, the smoke check and the benchmark's cpu_baseline leg can compare the HIP
// library against it.  The product (the HIP library and its Python binding) never
// includes, links, loads or calls anything in this directory, and this file shares
// no code, header, table or helper with the HIP sources.
//
// One traffic matrix at a time, plain nested loops over std::vector<int64_t>.
// No blocking, fusion or reordering beyond what each step states.
//
// Notation (paper, Section 4 and Appendix): S servers ("n"), G GPUs per server
// ("m"), N = S*G GPUs, GPU index g = a*G + i (server a, local index i, the order
// A_0, A_1, B_0, ... of Section 4.1).  traffic[g][h] = bytes GPU g sends to GPU h
// (row = sender, Section 4.1 "Example setup").  T[a][d] = total bytes server a ->
// server d, T[a][a] = 0 (Appendix, symbols).  B_up / B_out = per-GPU scale-up /
// scale-out bandwidth ("B_1", "B_2").
//
// Where the paper leaves a choice open, the reading taken is stated at the step.
// Every function below is pinned by tests/test_oracle_*.py (worked numbers from
// Section 4.1/4.2, Theorem 1, the stage-count bound of Section 4.4, invariants,
// and brute force on tiny clusters).  The particular sequence of matchings chosen
// by decompose() is one valid Birkhoff decomposition among many; the paper fixes
// its properties, not the sequence, so the sequence itself is "parity unpinned"
// by the paper and pinned only by the canonical rules written at decompose().

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <vector>

namespace {

typedef int64_t i64;

inline i64 at(const i64* m, int n, int r, int c) { return m[(size_t)r * n + c]; }

// ---------------------------------------------------------------------------
// Step 1 - server aggregation (Section 4.1 setup, Section 4.2 / Fig. 6, Appendix
// symbols): r_i(a,d) = bytes GPU (a,i) sends to server d; T[a][d] = sum_i r_i.
// GPU-diagonal entries (a GPU "sending to itself") use no link and are ignored.
// The intra-server tile (d == a) gives each GPU's intra-server outgoing and
// incoming bytes (the grey tiles of Fig. 5 / the S_i of the Appendix).
// Returns -1 if an off-diagonal entry is negative.
// ---------------------------------------------------------------------------
int aggregate(int S, int G, const i64* traffic, i64* T, i64* intra_out, i64* intra_in) {
    const int N = S * G;
    for (int g = 0; g < N; ++g)
        for (int h = 0; h < N; ++h)
            if (g != h && at(traffic, N, g, h) < 0) return -1;
    for (int a = 0; a < S; ++a)
        for (int d = 0; d < S; ++d) {
            i64 tot = 0;
            if (a != d)
                for (int i = 0; i < G; ++i)
                    for (int j = 0; j < G; ++j) tot += at(traffic, N, a * G + i, d * G + j);
            T[(size_t)a * S + d] = tot;
        }
    for (int a = 0; a < S; ++a)
        for (int i = 0; i < G; ++i) {
            i64 o = 0, in = 0;
            for (int j = 0; j < G; ++j)
                if (j != i) {
                    o += at(traffic, N, a * G + i, a * G + j);
                    in += at(traffic, N, a * G + j, a * G + i);
                }
            intra_out[a * G + i] = o;
            intra_in[a * G + i] = in;
        }
    return 0;
}

// ---------------------------------------------------------------------------
// Step 2 - sender balancing of one cross-server tile (Section 4.1 "Mitigating
// sender skew", Section 4.2 Step 1): heavy GPUs hand their excess to light GPUs
// until every GPU of the source server carries the same load for this destination
// server.  Input: the G tile row sums r.  Output: the G x G lane-routing tile X,
// X[i][k] = bytes of GPU i's traffic that leave on GPU k's NIC ("lane" k);
// k == i is what GPU i keeps, k != i is handed to GPU k over scale-up.
//
// Readings where the paper is silent:
//  * integer remainder: lane targets t_k = floor(T/G) + (k < T mod G ? 1 : 0);
//  * who gives to whom: surplus s_i = max(0, r_i - t_i), deficit d_k =
//    max(0, t_k - r_k); surplus is poured into deficit in ascending index order
//    (north-west-corner transport), which moves the minimum total, sum(s).
// ---------------------------------------------------------------------------
void rebalance_tile(int G, const i64* r, i64* X, i64* target) {
    i64 tot = 0;
    for (int i = 0; i < G; ++i) tot += r[i];
    const i64 q = tot / G, rho = tot % G;
    std::vector<i64> s(G), d(G);
    for (int k = 0; k < G; ++k) {
        target[k] = q + (k < rho ? 1 : 0);
        s[k] = std::max<i64>(0, r[k] - target[k]);
        d[k] = std::max<i64>(0, target[k] - r[k]);
    }
    for (int i = 0; i < G * G; ++i) X[i] = 0;
    for (int i = 0; i < G; ++i) X[i * G + i] = std::min(r[i], target[i]);
    int i = 0, k = 0;
    while (i < G && k < G) {
        if (s[i] == 0) { ++i; continue; }
        if (d[k] == 0) { ++k; continue; }
        const i64 mv = std::min(s[i], d[k]);
        X[i * G + k] += mv;
        s[i] -= mv;
        d[k] -= mv;
    }
}

// Whole lane-routing matrix X[N][N] (same tiling as traffic; intra tiles zero).
void rebalance(int S, int G, const i64* traffic, i64* X) {
    const int N = S * G;
    std::fill(X, X + (size_t)N * N, (i64)0);
    std::vector<i64> r(G), tile((size_t)G * G), tgt(G);
    for (int a = 0; a < S; ++a)
        for (int d = 0; d < S; ++d) {
            if (a == d) continue;
            for (int i = 0; i < G; ++i) {
                r[i] = 0;
                for (int j = 0; j < G; ++j) r[i] += at(traffic, N, a * G + i, d * G + j);
            }
            rebalance_tile(G, r.data(), tile.data(), tgt.data());
            for (int i = 0; i < G; ++i)
                for (int k = 0; k < G; ++k)
                    X[(size_t)(a * G + i) * N + d * G + k] = tile[i * G + k];
        }
}

// ---------------------------------------------------------------------------
// Step 3 - merged peer transfer and collapse (Section 4.1 "Mitigating receiver
// skew"; Section 4.2, Fig. 6): after balancing, GPU (a,k) sends its whole load for
// server d to the same-index GPU (d,k); the tile is a scalar matrix and becomes
// one server-level entry.  Reading: the entry is the per-lane byte count of the
// lane that gates the pair, Q[a][d] = ceil(T[a][d]/G) (= target of lane 0);
// Theorem 1's proof uses T_ij/m per GPU.  Q[a][a] = 0.
// ---------------------------------------------------------------------------
void collapse(int S, int G, const i64* T, i64* Q) {
    for (int a = 0; a < S; ++a)
        for (int d = 0; d < S; ++d) {
            const i64 t = at(T, S, a, d);
            Q[(size_t)a * S + d] = (a == d) ? 0 : (t + G - 1) / G;
        }
}

// ---------------------------------------------------------------------------
// Step 4 - embedding into a scaled doubly stochastic matrix (Section 4.4,
// "Adapting an arbitrary matrix to a valid form"): add a virtual matrix A >= 0 so
// that every row and column of Q + A sums to L = the heaviest row/column sum;
// only lighter rows/columns are raised, the bottleneck is untouched.
// Reading (the paper does not give the concrete A): first put as much as
// possible on the diagonal, A[a][a] = min(row deficit a, column deficit a) (the
// diagonal holds no real traffic); then pour the remaining row deficits into the
// remaining column deficits in ascending index order (north-west corner).
// Returns L.
// ---------------------------------------------------------------------------
i64 embed(int S, const i64* Q, i64* A) {
    std::vector<i64> dr(S, 0), dc(S, 0);
    i64 L = 0;
    for (int a = 0; a < S; ++a)
        for (int d = 0; d < S; ++d) {
            dr[a] += at(Q, S, a, d);
            dc[d] += at(Q, S, a, d);
        }
    for (int a = 0; a < S; ++a) L = std::max(L, std::max(dr[a], dc[a]));
    for (int a = 0; a < S; ++a) { dr[a] = L - dr[a]; dc[a] = L - dc[a]; }
    std::fill(A, A + (size_t)S * S, (i64)0);
    for (int a = 0; a < S; ++a) {
        const i64 m = std::min(dr[a], dc[a]);
        A[(size_t)a * S + a] = m;
        dr[a] -= m;
        dc[a] -= m;
    }
    int a = 0, d = 0;
    while (a < S && d < S) {
        if (dr[a] == 0) { ++a; continue; }
        if (dc[d] == 0) { ++d; continue; }
        const i64 mv = std::min(dr[a], dc[d]);
        A[(size_t)a * S + d] += mv;
        dr[a] -= mv;
        dc[d] -= mv;
    }
    return L;
}

// ---------------------------------------------------------------------------
// Step 5 - Birkhoff decomposition (Section 4.4 "Birkhoff's decomposition:
// overview"; Section 4.2): repeatedly take a perfect matching on the support of
// the residual R = Q + A, subtract it with the weight of its smallest matched
// entry, repeat; the residual stays scaled doubly stochastic.  Each matching is
// one scale-out stage; virtual bytes are never sent, so a stage may be a partial
// permutation with respect to real traffic.
//
// The paper fixes neither the matching routine (Hungarian is its example), nor
// the stage weight, nor how a cell holding both real and virtual bytes is
// consumed.  Canonical rules used here:
//  * matching = augmenting paths found by a level-synchronous breadth-first
//    search from one unmatched row; within a level a newly reached column takes
//    as parent the lowest-numbered frontier row with a positive cell; the search
//    stops at the first level that reaches an unmatched column and takes the
//    lowest-numbered such column;
//  * the first matching is built by augmenting rows 0..S-1 in order;
//  * stage weight c = smallest residual among matched cells;
//  * in a cell, real bytes are consumed before virtual bytes; a row whose matched
//    cell has no real bytes left is idle in that stage (destination -1);
//  * after a stage only rows whose matched cell reached zero are unmatched; all
//    of them are unmatched first, then re-augmented in ascending row order.
//
// Outputs: stages[s*S + a] = destination server of server a in stage s or -1,
// bytes[s*S + a] = real per-lane bytes it sends in that stage.  Returns the
// number of stages K, -2 if more than `cap` stages would be needed, -3 if no
// augmenting path exists (impossible for a doubly stochastic residual).
// ---------------------------------------------------------------------------
struct Matcher {
    int S;
    const std::vector<i64>& R;
    std::vector<int> mr, mc;  // row -> matched column, column -> matched row
    i64 thr;                  // a cell is an edge while it holds at least thr bytes (1: the support)
    Matcher(int S_, const std::vector<i64>& R_, i64 thr_ = 1)
        : S(S_), R(R_), mr(S_, -1), mc(S_, -1), thr(thr_) {}

    bool augment(int r0) {
        std::vector<char> visited(S, 0), inF(S, 0);
        std::vector<int> parent(S, -1);
        inF[r0] = 1;
        for (;;) {
            std::vector<int> fresh;
            for (int d = 0; d < S; ++d) {
                if (visited[d]) continue;
                for (int a = 0; a < S; ++a)
                    if (inF[a] && R[(size_t)a * S + d] >= thr) {
                        parent[d] = a;  // lowest-numbered frontier row
                        fresh.push_back(d);
                        break;
                    }
            }
            if (fresh.empty()) return false;
            for (int d : fresh) visited[d] = 1;
            int dstar = -1;
            for (int d : fresh)
                if (mc[d] < 0) { dstar = d; break; }  // fresh is ascending
            if (dstar >= 0) {
                int d = dstar;
                for (;;) {
                    const int a = parent[d];
                    const int prev = mr[a];
                    mr[a] = d;
                    mc[d] = a;
                    if (a == r0) break;
                    d = prev;
                }
                return true;
            }
            std::fill(inF.begin(), inF.end(), 0);
            for (int d : fresh) inF[mc[d]] = 1;
        }
    }
};

// One stage from a perfect matching mr (row -> column): the weight is the smallest
// matched residual; every matched cell loses it, real bytes first.  Returns the weight.
i64 take_stage(int S, const std::vector<int>& mr, std::vector<i64>& R, std::vector<i64>& Rreal,
               int32_t* stage_row, i64* bytes_row) {
    i64 c = R[(size_t)0 * S + mr[0]];
    for (int a = 1; a < S; ++a) c = std::min(c, R[(size_t)a * S + mr[a]]);
    for (int a = 0; a < S; ++a) {
        const int d = mr[a];
        const i64 real = std::min(c, Rreal[(size_t)a * S + d]);
        Rreal[(size_t)a * S + d] -= real;
        R[(size_t)a * S + d] -= c;
        stage_row[a] = real > 0 ? d : -1;
        bytes_row[a] = real;
    }
    return c;
}

int decompose(int S, const i64* Q, const i64* A, int cap, int32_t* stages, i64* bytes) {
    std::vector<i64> R((size_t)S * S), Rreal((size_t)S * S);
    std::vector<i64> rowsum(S, 0);
    for (int a = 0; a < S; ++a)
        for (int d = 0; d < S; ++d) {
            R[(size_t)a * S + d] = at(Q, S, a, d) + at(A, S, a, d);
            Rreal[(size_t)a * S + d] = at(Q, S, a, d);
            rowsum[a] += R[(size_t)a * S + d];
        }
    i64 Lrem = S > 0 ? rowsum[0] : 0;
    if (Lrem == 0) return 0;

    Matcher M(S, R);
    for (int r0 = 0; r0 < S; ++r0)
        if (!M.augment(r0)) return -3;

    int s = 0;
    for (;;) {
        if (s >= cap) return -2;
        const i64 c = take_stage(S, M.mr, R, Rreal, stages + (size_t)s * S, bytes + (size_t)s * S);
        Lrem -= c;
        ++s;
        if (Lrem == 0) return s;
        std::vector<int> freed;
        for (int a = 0; a < S; ++a)
            if (R[(size_t)a * S + M.mr[a]] == 0) freed.push_back(a);
        for (int a : freed) { M.mc[M.mr[a]] = -1; M.mr[a] = -1; }
        for (int a : freed)
            if (!M.augment(a)) return -3;
    }
}

// ---------------------------------------------------------------------------
// Variant of step 5 with fewer, larger stages (Section 4.4 "Number of stages":
// fewer stages are preferable since each costs a synchronisation, and the minimum
// is NP-hard to find; the paper itself stops at "any valid decomposition").  The
// greedy rule taken here, which is not the paper's: every stage removes as much
// weight as one stage can, i.e. its matching is a bottleneck assignment of the
// residual - a perfect matching whose smallest cell is as large as possible.
//
//  * bottleneck value t* of R = the largest t such that the cells with R >= t
//    contain a perfect matching (equivalently the maximum over all perfect
//    matchings of their smallest cell).  t* is one of the cell values, and a
//    perfect matching that exists for t exists for every smaller t, so a binary
//    search over the sorted distinct values is exact; existence is decided by a
//    plain depth-first augmenting search (Kuhn), which shares nothing with the
//    canonical Matcher;
//  * the stage's matching = the canonical matching (rules at decompose()) of the
//    graph {R >= t*}, built from nothing by augmenting rows 0..S-1 in order; its
//    smallest cell is t* and that is the stage weight;
//  * real bytes before virtual bytes, idle rows, outputs, return values: as in
//    decompose().
// The residual only shrinks, so the stage weights never increase; the stage-count
// bound of Section 4.4 holds for any choice of matchings.  Which matchings come
// out is this variant's own rule ("parity unpinned" by the paper); the bottleneck
// value is pinned by brute force over all permutations and by a library matching.
// ---------------------------------------------------------------------------
bool kuhn_try(int S, const std::vector<i64>& R, i64 t, int a, std::vector<char>& seen,
              std::vector<int>& owner) {
    for (int d = 0; d < S; ++d) {
        if (R[(size_t)a * S + d] < t || seen[d]) continue;
        seen[d] = 1;
        if (owner[d] < 0 || kuhn_try(S, R, t, owner[d], seen, owner)) {
            owner[d] = a;
            return true;
        }
    }
    return false;
}

bool has_perfect_matching(int S, const std::vector<i64>& R, i64 t) {
    std::vector<int> owner(S, -1);
    for (int a = 0; a < S; ++a) {
        std::vector<char> seen(S, 0);
        if (!kuhn_try(S, R, t, a, seen, owner)) return false;
    }
    return true;
}

// 0 if even the support of R holds no perfect matching
i64 bottleneck_value(int S, const std::vector<i64>& R) {
    std::vector<i64> vals;
    for (i64 v : R)
        if (v > 0) vals.push_back(v);
    std::sort(vals.begin(), vals.end());
    vals.erase(std::unique(vals.begin(), vals.end()), vals.end());
    i64 best = 0;
    int lo = 0, hi = (int)vals.size() - 1;
    while (lo <= hi) {
        const int mid = lo + (hi - lo) / 2;
        if (has_perfect_matching(S, R, vals[mid])) {
            best = vals[mid];
            lo = mid + 1;
        } else {
            hi = mid - 1;
        }
    }
    return best;
}

int decompose_bottleneck(int S, const i64* Q, const i64* A, int cap, int32_t* stages, i64* bytes) {
    std::vector<i64> R((size_t)S * S), Rreal((size_t)S * S);
    i64 Lrem = 0;
    for (int a = 0; a < S; ++a)
        for (int d = 0; d < S; ++d) {
            R[(size_t)a * S + d] = at(Q, S, a, d) + at(A, S, a, d);
            Rreal[(size_t)a * S + d] = at(Q, S, a, d);
            if (a == 0) Lrem += R[(size_t)a * S + d];
        }
    int s = 0;
    while (Lrem > 0) {
        if (s >= cap) return -2;
        const i64 t = bottleneck_value(S, R);
        if (t <= 0) return -3;
        Matcher M(S, R, t);
        for (int r0 = 0; r0 < S; ++r0)
            if (!M.augment(r0)) return -3;
        const i64 c = take_stage(S, M.mr, R, Rreal, stages + (size_t)s * S, bytes + (size_t)s * S);
        Lrem -= c;
        ++s;
    }
    return s;
}

// ---------------------------------------------------------------------------
// Step 6 - analytical completion time (Section 5.4 simulator: sum of per-step
// size/bandwidth, wake-up delay taken as 0 because the paper gives no value;
// Appendix, Theorems 1 and 2: balance -> intra-server portion -> Birkhoff stages
// -> last stage's redistribution, t_FAST = t0 + t1 + t2 + t3).  The Appendix
// prints worst-case values of the four terms; here the same four terms are
// evaluated on the actual plan:
//   t0 = max over GPUs of max(bytes it hands off, bytes it is handed) / B_up
//   t1 = max over GPUs of max(intra-server bytes out, in) / B_up   (serialised
//        after balancing as in the Appendix formula)
//   t2 = (sum over stages of c_s) / B_out, c_s = largest per-lane real bytes of
//        stage s
//   t3 = (G-1) * max_s c_s / B_up  (stages run in ascending size, so the last one
//        is the largest; a destination GPU may have to forward all it received
//        to one GPU: the (m-1) l_i / B_1 of the proof of Theorem 2.  The printed
//        t3 drops the (m-1) factor that the proof's own step (i) carries; the
//        factor is kept here.)
//   if B_up < (G-1) B_out the redistributions no longer hide under the next
//   stage; with sizes sorted ascending l_0 <= l_1 <= ... the exposed part
//   sum_{i>=1} max(0, (G-1) l_{i-1}/B_up - l_i/B_out) is added (t_exc).  Reading:
//   the proof's execution with a synchronisation between pipeline steps - step i
//   moves stage i over scale-out while stage i-1 is redistributed, and ends when
//   both have ended - so every overhang delays everything after it and an overhang
//   is never absorbed by a later, longer stage (pipeline_time() below is the
//   free-running pipeline of Section 4.3, where it can be).
//   t_opt = max(max row sum, max column sum of T) / (G * B_out)   (Theorem 1).
//   wake-up delay (Section 5.4: every transfer step costs a fixed link wake-up
//   delay plus size/bandwidth): `delay` seconds are added once per executed step;
//   the steps are the balance (if anything is handed off), the intra-server
//   portion (if any), each of the K stages, and the last redistribution (if G > 1
//   and K > 0).  The paper gives no value for it; 0 reproduces the Appendix.
// out4 = {T_pred, t0, t2, t_opt}; extra3 (optional) = {t1, t3, t_exc}.
// ---------------------------------------------------------------------------
void cost(int S, int G, double bw_up, double bw_out, double delay, const i64* T, const i64* X,
          const i64* intra_out, const i64* intra_in, int K, const i64* bytes, double* out4,
          double* extra3) {
    const int N = S * G;
    i64 bal = 0;
    for (int a = 0; a < S; ++a)
        for (int i = 0; i < G; ++i) {
            i64 handed_off = 0, handed_in = 0;
            for (int d = 0; d < S; ++d) {
                if (d == a) continue;
                for (int k = 0; k < G; ++k) {
                    if (k == i) continue;
                    handed_off += at(X, N, a * G + i, d * G + k);  // i's bytes leaving on lane k
                    handed_in += at(X, N, a * G + k, d * G + i);   // k's bytes arriving for lane i
                }
            }
            bal = std::max(bal, std::max(handed_off, handed_in));
        }
    i64 intra = 0;
    for (int g = 0; g < N; ++g) intra = std::max(intra, std::max(intra_out[g], intra_in[g]));

    std::vector<i64> c(K > 0 ? K : 0);
    i64 csum = 0, cmax = 0;
    for (int s = 0; s < K; ++s) {
        i64 m = 0;
        for (int a = 0; a < S; ++a) m = std::max(m, bytes[(size_t)s * S + a]);
        c[s] = m;
        csum += m;
        cmax = std::max(cmax, m);
    }
    i64 big = 0;
    for (int a = 0; a < S; ++a) {
        i64 rs = 0, cs = 0;
        for (int d = 0; d < S; ++d) { rs += at(T, S, a, d); cs += at(T, S, d, a); }
        big = std::max(big, std::max(rs, cs));
    }
    const double t0 = (double)bal / bw_up;
    const double t1 = (double)intra / bw_up;
    const double t2 = (double)csum / bw_out;
    const double t3 = (double)((i64)(G - 1) * cmax) / bw_up;
    double texc = 0.0;
    if (bw_up < (double)(G - 1) * bw_out) {
        std::sort(c.begin(), c.end());
        for (int i = 1; i < K; ++i) {
            const double redis = (double)((i64)(G - 1) * c[i - 1]) / bw_up;
            const double next = (double)c[i] / bw_out;
            if (redis > next) texc += redis - next;
        }
    }
    double tp = t0 + t1;
    tp = tp + t2;
    tp = tp + t3;
    tp = tp + texc;
    const int steps = (bal > 0 ? 1 : 0) + (intra > 0 ? 1 : 0) + (K > 0 ? K : 0) +
                      ((i64)(G - 1) * cmax > 0 ? 1 : 0);
    tp = tp + delay * (double)steps;
    out4[0] = tp;
    out4[1] = t0;
    out4[2] = t2;
    out4[3] = (double)big / ((double)G * bw_out);
    if (extra3) { extra3[0] = t1; extra3[1] = t3; extra3[2] = texc; }
}

// ---------------------------------------------------------------------------
// SpreadOut baseline (Section 4.2 "SpreadOut: one-to-one but not optimal";
// Section 5.4 compares FAST with it in simulation): stage i pairs endpoint s with
// endpoint (s+i) mod n for i = 1..n-1, every stage lasts as long as its largest
// transfer, so the completion time is the sum over shifted diagonals of the
// largest entry's transfer time (plus the wake-up delay per non-empty stage).
//   out2[0]: SpreadOut over the N GPUs on the raw matrix, a pair inside a server
//            moving at B_up and a pair across servers at B_out;
//   out2[1]: SpreadOut over the S servers on the balanced per-lane matrix Q (the
//            comparison of Fig. 7: same balancing as FAST, shifted diagonals
//            instead of Birkhoff stages).
// Returns -1 if an off-diagonal entry is negative.
// ---------------------------------------------------------------------------
int spreadout(int S, int G, double bw_up, double bw_out, double delay, const i64* traffic,
              double* out2) {
    const int N = S * G;
    std::vector<i64> T((size_t)S * S), Q((size_t)S * S), io(N), ii(N);
    if (aggregate(S, G, traffic, T.data(), io.data(), ii.data()) != 0) return -1;
    double tg = 0.0;
    for (int i = 1; i < N; ++i) {
        i64 up = 0, out = 0;
        for (int g = 0; g < N; ++g) {
            const int h = (g + i) % N;
            const i64 v = at(traffic, N, g, h);
            if (g / G == h / G) up = std::max(up, v); else out = std::max(out, v);
        }
        if (up > 0 || out > 0) {
            const double a = (double)up / bw_up, b = (double)out / bw_out;
            tg = tg + (delay + (a > b ? a : b));
        }
    }
    collapse(S, G, T.data(), Q.data());
    double ts = 0.0;
    for (int i = 1; i < S; ++i) {
        i64 m = 0;
        for (int a = 0; a < S; ++a) m = std::max(m, at(Q.data(), S, a, (a + i) % S));
        if (m > 0) ts = ts + (delay + (double)m / bw_out);
    }
    out2[0] = tg;
    out2[1] = ts;
    return 0;
}

// ---------------------------------------------------------------------------
// Execution order of the stages (Appendix, proof of Theorem 2: the stages are
// sorted in ascending order of their transfer size and executed in that order, so
// that each stage's redistribution hides under the next, larger, stage).  The
// weight of stage s is its largest per-lane byte count; order[] lists the stage
// indices by ascending weight, equal weights in extraction order.
// ---------------------------------------------------------------------------
void stage_order(int S, int K, const i64* bytes, int32_t* order) {
    std::vector<i64> c(K > 0 ? K : 0);
    for (int s = 0; s < K; ++s) {
        i64 m = 0;
        for (int a = 0; a < S; ++a) m = std::max(m, bytes[(size_t)s * S + a]);
        c[s] = m;
    }
    for (int s = 0; s < K; ++s) order[s] = s;
    // insertion sort: plainly stable
    for (int i = 1; i < K; ++i) {
        const int32_t x = order[i];
        int j = i - 1;
        while (j >= 0 && c[order[j]] > c[x]) { order[j + 1] = order[j]; --j; }
        order[j + 1] = x;
    }
}

// ---------------------------------------------------------------------------
// Traffic-matrix construction (Section 5 "Integration into MoE systems": the
// All-Gather of per-expert token counts that MoE frameworks already perform gives
// every rank counts[src][e] = tokens GPU src routes to expert e, "from which the
// full traffic matrix can be constructed"): traffic[src][h] = token_bytes * sum of
// counts[src][e] over the experts e placed on GPU h.  The diagonal holds what
// stays on the GPU (the scheduler ignores it).  Returns -1 if a count is negative
// or an expert is mapped outside 0..N-1 (traffic is then unspecified).
// ---------------------------------------------------------------------------
int build_traffic(int N, int E, const i64* counts, const int32_t* expert_to_gpu, i64 token_bytes,
                  i64* traffic) {
    for (int e = 0; e < E; ++e)
        if (expert_to_gpu[e] < 0 || expert_to_gpu[e] >= N) return -1;
    for (int src = 0; src < N; ++src) {
        for (int h = 0; h < N; ++h) traffic[(size_t)src * N + h] = 0;
        for (int e = 0; e < E; ++e) {
            const i64 c = counts[(size_t)src * E + e];
            if (c < 0) return -1;
            traffic[(size_t)src * N + expert_to_gpu[e]] += c * token_bytes;
        }
    }
    return 0;
}

// ---------------------------------------------------------------------------
// Which bytes travel where (Section 4.1 "Redistribution", Section 4.2 Step 3
// "Per-stage redistribution"): after a stage's scale-out transfer the data sits on
// the right server but possibly on the wrong GPU, and is forwarded over scale-up
// from the proxy GPU (d,k) that received it to its destination GPU (d,j).
//
// The paper does not say which of a GPU's bytes are the ones handed to another
// lane, nor in which order a lane sends what it holds, so a byte-identity policy is
// fixed here:
//  * the bytes GPU (a,i) holds for server d form one region, ordered by
//    destination GPU: traffic[(a,i)][(d,0)] bytes for (d,0), then those for (d,1),
//    ... ;
//  * balancing: the GPU keeps the head of its region (as many bytes as it sends on
//    its own lane) and hands off the tail; the tail is cut into the pieces of
//    rebalance_tile() in ascending receiver index;
//  * lane k's send queue for server d is what GPU (a,k) kept, followed by the
//    pieces it was handed in ascending donor index;
//  * every stage in which a sends to d takes the next bytes[s][a] bytes from the
//    front of each lane's queue (a lane whose queue is one byte shorter, because
//    the tile total is not a multiple of G, runs out one byte early).
// lane_queues() builds the G queues of one tile as runs of equal destination.
// ---------------------------------------------------------------------------
struct Run { int dest; i64 len; };
struct Queue {
    std::vector<Run> runs;
    size_t head = 0;       // first run not yet fully taken
    i64 used = 0;          // bytes already taken from runs[head]
    void push(const Run& r) { if (r.len > 0) runs.push_back(r); }
    // Removes up to n bytes from the front and appends them to `out`.
    void take(i64 n, Queue* out) {
        while (n > 0 && head < runs.size()) {
            const i64 avail = runs[head].len - used;
            const i64 mv = std::min(avail, n);
            out->push({runs[head].dest, mv});
            used += mv;
            n -= mv;
            if (used == runs[head].len) { ++head; used = 0; }
        }
    }
};

// tile: G x G traffic tile of one ordered server pair, tile[i*G+j] = bytes (a,i) -> (d,j).
void lane_queues(int G, const i64* tile, std::vector<Queue>* queue) {
    std::vector<Queue> region(G);
    std::vector<i64> r(G, 0);
    i64 tot = 0;
    for (int i = 0; i < G; ++i)
        for (int j = 0; j < G; ++j) {
            region[i].push({j, tile[i * G + j]});
            r[i] += tile[i * G + j];
            tot += tile[i * G + j];
        }
    const i64 q = tot / G, rho = tot % G;
    std::vector<i64> s(G), d(G);
    queue->assign(G, Queue());
    for (int k = 0; k < G; ++k) {
        const i64 target = q + (k < rho ? 1 : 0);
        s[k] = std::max<i64>(0, r[k] - target);
        d[k] = std::max<i64>(0, target - r[k]);
        region[k].take(std::min(r[k], target), &(*queue)[k]);   // the head stays on lane k
    }
    // the tails are poured in the order of rebalance_tile(): lowest donor into lowest taker
    for (int i = 0, k = 0;;) {
        while (i < G && s[i] == 0) ++i;
        while (k < G && d[k] == 0) ++k;
        if (i == G || k == G) break;
        const i64 piece = std::min(s[i], d[k]);
        region[i].take(piece, &(*queue)[k]);
        s[i] -= piece;
        d[k] -= piece;
    }
}

// Plays the K stages in execution order (order[e] = e-th stage to run; NULL = the
// order they were extracted in) and records, per stage s and source server a:
//   offsets[s][a]    per-lane bytes a had already sent to stages[s][a] before s
//                    (0 where a is idle in s);
//   redis_bytes[s]   scale-up volume of the stage's redistribution = the largest,
//                    over the GPUs of all receiving servers, of max(bytes the GPU
//                    forwards to other GPUs, bytes it is forwarded by others);
//   for each selected stage sel[q], sel_out[q][d][k][j] = bytes that arrived at
//   server d on lane k in that stage and belong to GPU (d,j) (zero tile if no
//   server sends to d in that stage).
void redistribution(int S, int G, const i64* traffic, int K, const int32_t* stages, const i64* bytes,
                    const int32_t* order, i64* offsets, i64* redis_bytes, int n_sel,
                    const int32_t* sel, i64* sel_out) {
    const int N = S * G;
    std::vector<std::vector<Queue>> queues((size_t)S * S);
    std::vector<i64> sent((size_t)S * S, 0), tile((size_t)G * G), M((size_t)G * G);
    for (int a = 0; a < S; ++a)
        for (int d = 0; d < S; ++d) {
            if (a == d) continue;
            for (int i = 0; i < G; ++i)
                for (int j = 0; j < G; ++j) tile[i * G + j] = at(traffic, N, a * G + i, d * G + j);
            lane_queues(G, tile.data(), &queues[(size_t)a * S + d]);
        }
    if (n_sel > 0) std::fill(sel_out, sel_out + (size_t)n_sel * S * G * G, (i64)0);
    for (int e = 0; e < K; ++e) {
        const int s = order ? order[e] : e;
        i64 worst = 0;
        for (int a = 0; a < S; ++a) {
            const int d = stages[(size_t)s * S + a];
            offsets[(size_t)s * S + a] = 0;
            if (d < 0) continue;
            const i64 len = bytes[(size_t)s * S + a];
            offsets[(size_t)s * S + a] = sent[(size_t)a * S + d];
            sent[(size_t)a * S + d] += len;
            std::fill(M.begin(), M.end(), (i64)0);
            for (int k = 0; k < G; ++k) {
                Queue got;
                queues[(size_t)a * S + d][k].take(len, &got);
                for (const Run& run : got.runs) M[k * G + run.dest] += run.len;
            }
            for (int g = 0; g < G; ++g) {
                i64 fwd = 0, recv = 0;
                for (int o = 0; o < G; ++o) {
                    if (o == g) continue;
                    fwd += M[g * G + o];     // arrived at g, belongs to o
                    recv += M[o * G + g];    // arrived at o, belongs to g
                }
                worst = std::max(worst, std::max(fwd, recv));
            }
            for (int q = 0; q < n_sel; ++q)
                if (sel[q] == s)
                    std::copy(M.begin(), M.end(), sel_out + ((size_t)q * S + d) * G * G);
        }
        redis_bytes[s] = worst;
    }
}

// ---------------------------------------------------------------------------
// Completion time of the overlapped pipeline (Section 4.3 "Pipeline structure"):
// balancing runs first; then the scale-out stages run back to back; the
// intra-server portion of the All-to-All runs on the scale-up fabric alongside the
// first stage; stage i's redistribution starts when stage i's scale-out has ended
// and the scale-up fabric is free (it is used by one thing at a time: the
// intra-server portion, then the redistributions in stage order), overlapping
// the following stages; the last redistribution has nothing to hide under.
// Every step that moves bytes costs the wake-up delay plus bytes / bandwidth
// (Section 5.4).  weight[e] / redis[e] are the e-th executed stage's per-lane
// scale-out bytes and its redistribution's scale-up bytes.
//   out2[0] = completion time, out2[1] = time at which the last scale-out ends.
// ---------------------------------------------------------------------------
void pipeline_time(double bw_up, double bw_out, double delay, i64 bal, i64 intra, int K,
                   const i64* weight, const i64* redis, double* out2) {
    double t = 0.0;
    if (bal > 0) t = delay + (double)bal / bw_up;
    double out_end = t, up_free = t;
    if (intra > 0) up_free = t + (delay + (double)intra / bw_up);
    for (int e = 0; e < K; ++e) {
        out_end = out_end + (delay + (double)weight[e] / bw_out);
        if (redis[e] > 0) {
            const double start = std::max(out_end, up_free);
            up_free = start + (delay + (double)redis[e] / bw_up);
        }
    }
    out2[0] = std::max(out_end, up_free);
    out2[1] = out_end;
}

}  // namespace

// ---------------------------------------------------------------------------
// C entry points (loaded with ctypes by the tests).  All pointers are host
// memory owned by the caller.
// ---------------------------------------------------------------------------
extern "C" {

int oracle_aggregate(int S, int G, const int64_t* traffic, int64_t* T, int64_t* intra_out,
                     int64_t* intra_in) {
    return aggregate(S, G, traffic, T, intra_out, intra_in);
}

void oracle_rebalance_tile(int G, const int64_t* r, int64_t* X, int64_t* target) {
    rebalance_tile(G, r, X, target);
}

void oracle_rebalance(int S, int G, const int64_t* traffic, int64_t* X) {
    rebalance(S, G, traffic, X);
}

void oracle_collapse(int S, int G, const int64_t* T, int64_t* Q) { collapse(S, G, T, Q); }

int64_t oracle_embed(int S, const int64_t* Q, int64_t* A) { return embed(S, Q, A); }

int oracle_decompose(int S, const int64_t* Q, const int64_t* A, int cap, int32_t* stages,
                     int64_t* bytes) {
    return decompose(S, Q, A, cap, stages, bytes);
}

int oracle_decompose_bottleneck(int S, const int64_t* Q, const int64_t* A, int cap,
                                int32_t* stages, int64_t* bytes) {
    return decompose_bottleneck(S, Q, A, cap, stages, bytes);
}

int64_t oracle_bottleneck_value(int S, const int64_t* R) {
    return bottleneck_value(S, std::vector<i64>(R, R + (size_t)S * S));
}

void oracle_cost(int S, int G, double bw_up, double bw_out, double delay, const int64_t* T,
                 const int64_t* X, const int64_t* intra_out, const int64_t* intra_in, int K,
                 const int64_t* bytes, double* out4, double* extra3) {
    cost(S, G, bw_up, bw_out, delay, T, X, intra_out, intra_in, K, bytes, out4, extra3);
}

void oracle_stage_order(int S, int K, const int64_t* bytes, int32_t* order) {
    stage_order(S, K, bytes, order);
}

int oracle_build_traffic(int N, int E, const int64_t* counts, const int32_t* expert_to_gpu,
                         int64_t token_bytes, int64_t* traffic) {
    return build_traffic(N, E, counts, expert_to_gpu, token_bytes, traffic);
}

int oracle_spreadout(int S, int G, double bw_up, double bw_out, double delay,
                     const int64_t* traffic, double* out2) {
    return spreadout(S, G, bw_up, bw_out, delay, traffic, out2);
}

// Whole path for one matrix.  stages/bytes hold `cap` stage rows of S entries;
// rows >= K are left untouched.  *num_stages = K >= 0, -1 (negative entry),
// -2 (cap exceeded), -3 (internal).  Q_out / A_out (S*S each) may be NULL.
// bottleneck != 0 takes the stages from decompose_bottleneck() instead of decompose().
int oracle_synthesize(int S, int G, double bw_up, double bw_out, double delay,
                      const int64_t* traffic,
                      int64_t* X, int32_t* stages, int64_t* bytes, int cap, int32_t* num_stages,
                      double* out4, double* extra3, int64_t* Q_out, int64_t* A_out,
                      int bottleneck) {
    const int N = S * G;
    std::vector<i64> T((size_t)S * S), Q((size_t)S * S), A((size_t)S * S), io(N), ii(N);
    if (aggregate(S, G, traffic, T.data(), io.data(), ii.data()) != 0) {
        *num_stages = -1;
        return 0;
    }
    rebalance(S, G, traffic, X);
    collapse(S, G, T.data(), Q.data());
    embed(S, Q.data(), A.data());
    const int K = bottleneck ? decompose_bottleneck(S, Q.data(), A.data(), cap, stages, bytes)
                             : decompose(S, Q.data(), A.data(), cap, stages, bytes);
    *num_stages = K;
    if (Q_out) std::memcpy(Q_out, Q.data(), sizeof(i64) * S * S);
    if (A_out) std::memcpy(A_out, A.data(), sizeof(i64) * S * S);
    if (K < 0) return 0;
    cost(S, G, bw_up, bw_out, delay, T.data(), X, io.data(), ii.data(), K, bytes, out4, extra3);
    return 0;
}

void oracle_redistribution(int S, int G, const int64_t* traffic, int K, const int32_t* stages,
                           const int64_t* bytes, const int32_t* order, int64_t* offsets,
                           int64_t* redis_bytes, int n_sel, const int32_t* sel, int64_t* sel_out) {
    redistribution(S, G, traffic, K, stages, bytes, order, offsets, redis_bytes, n_sel, sel, sel_out);
}

// Pipelined completion time of a plan.  X, intra_out, intra_in as for oracle_cost;
// bytes = the K stage rows; order = execution order or NULL; redis = per-stage (indexed
// by stage, not by position) redistribution bytes, or NULL for the worst case of the
// Appendix, (G-1) * stage weight.
void oracle_pipeline_time(int S, int G, double bw_up, double bw_out, double delay, const int64_t* X,
                          const int64_t* intra_out, const int64_t* intra_in, int K,
                          const int64_t* bytes, const int32_t* order, const int64_t* redis,
                          double* out2) {
    const int N = S * G;
    i64 bal = 0;
    for (int a = 0; a < S; ++a)
        for (int i = 0; i < G; ++i) {
            i64 handed_off = 0, handed_in = 0;
            for (int d = 0; d < S; ++d) {
                if (d == a) continue;
                for (int k = 0; k < G; ++k) {
                    if (k == i) continue;
                    handed_off += at(X, N, a * G + i, d * G + k);
                    handed_in += at(X, N, a * G + k, d * G + i);
                }
            }
            bal = std::max(bal, std::max(handed_off, handed_in));
        }
    i64 intra = 0;
    for (int g = 0; g < N; ++g) intra = std::max(intra, std::max(intra_out[g], intra_in[g]));
    std::vector<i64> w(K > 0 ? K : 0), rb(K > 0 ? K : 0);
    for (int e = 0; e < K; ++e) {
        const int s = order ? order[e] : e;
        i64 m = 0;
        for (int a = 0; a < S; ++a) m = std::max(m, bytes[(size_t)s * S + a]);
        w[e] = m;
        rb[e] = redis ? redis[s] : (i64)(G - 1) * m;
    }
    pipeline_time(bw_up, bw_out, delay, bal, intra, K, w.data(), rb.data(), out2);
}

}  // extern "C"
