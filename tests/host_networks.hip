// Host-side check of the compare-exchange networks and the slot search used by the
// kernels (they are __host__ __device__): exhaustive 0-1 inputs where feasible, random
// floats otherwise.  Prints "ok" and exits 0 on success.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "../paper_1412_4944_amd/csrc/device_utils.h"

using namespace sbo;

static int fails = 0;
#define CHECK(c) do { if (!(c)) { if (fails++ < 10) std::printf("FAIL %s line %d\n", #c, __LINE__); } } while (0)

template <int N> static void test_sort() {
    const unsigned long long lim = N <= 16 ? (1ull << N) : 0;
    for (unsigned long long b = 0; b < lim; ++b) {
        float v[N];
        for (int i = 0; i < N; ++i) v[i] = (b >> i) & 1;
        bitonic_sort_desc<N>(v);
        for (int i = 1; i < N; ++i) CHECK(v[i - 1] >= v[i]);
    }
    std::mt19937 g(N);
    std::normal_distribution<float> d;
    for (int rep = 0; rep < 2000; ++rep) {
        float v[N], w[N];
        for (int i = 0; i < N; ++i) v[i] = w[i] = d(g);
        bitonic_sort_desc<N>(v);
        std::sort(w, w + N, [](float a, float b) { return a > b; });
        for (int i = 0; i < N; ++i) CHECK(v[i] == w[i]);
    }
}

// the three-input insertion networks: exhaustive 0-1 inputs (a network of min / max / median
// operations that sorts every 0-1 input sorts every input) and random floats
template <int N> static void test_insertion() {
    for (unsigned long long b = 0; b < (1ull << N); ++b) {
        float v[N];
        int ones = 0;
        for (int i = 0; i < N; ++i) { v[i] = (b >> i) & 1; ones += (b >> i) & 1; }
        insertion_sort_desc<N>(v);
        for (int i = 0; i < N; ++i) CHECK(v[i] == (i < ones ? 1.f : 0.f));
    }
    std::mt19937 g(300 + N);
    std::normal_distribution<float> d;
    for (int rep = 0; rep < 2000; ++rep) {
        float v[N], w[N];
        for (int i = 0; i < N; ++i) v[i] = w[i] = (rep & 3) == 0 ? float(int(d(g) * 2)) : d(g);   // with ties
        insertion_sort_desc<N>(v);
        std::sort(w, w + N, [](float a, float b) { return a > b; });
        for (int i = 0; i < N; ++i) CHECK(v[i] == w[i]);
    }
}

static void test_sort8() {
    for (unsigned b = 0; b < 256; ++b) {
        float v[8];
        for (int i = 0; i < 8; ++i) v[i] = (b >> i) & 1;
        sort8_desc(v);
        for (int i = 1; i < 8; ++i) CHECK(v[i - 1] >= v[i]);
    }
}

template <int N> static void test_merge() {
    std::mt19937 g(100 + N);
    std::normal_distribution<float> d;
    for (int rep = 0; rep < 2000; ++rep) {
        // bitonic input: descending run followed by ascending run (any split)
        float v[N], w[N];
        int cut = g() % (N + 1);
        for (int i = 0; i < N; ++i) w[i] = d(g);
        std::sort(w, w + cut, [](float a, float b) { return a > b; });
        std::sort(w + cut, w + N);
        for (int i = 0; i < N; ++i) v[i] = w[i];
        bitonic_merge_desc<N>(v);
        std::sort(w, w + N, [](float a, float b) { return a > b; });
        for (int i = 0; i < N; ++i) CHECK(v[i] == w[i]);
    }
}

template <int NV, int L> static void test_top() {
    std::mt19937 g(1000 + NV * 17 + L);
    std::normal_distribution<float> d;
    for (int rep = 0; rep < 4000; ++rep) {
        float x[NV], w[NV], out[L];
        const bool binary = rep & 1;
        for (int i = 0; i < NV; ++i) x[i] = w[i] = binary ? float(g() & 1) : d(g) * d(g);
        top_sorted<NV, L>(x, out);
        std::sort(w, w + NV, [](float a, float b) { return a > b; });
        for (int i = 0; i < L; ++i) CHECK(out[i] == w[i]);
    }
}

// top-S of the union of two lanes' lists, as the kernels merge them
template <int S> static void test_pair_fold() {
    std::mt19937 g(5000 + S);
    std::normal_distribution<float> d;
    for (int rep = 0; rep < 4000; ++rep) {
        float a[S], b[S], c[S];
        std::vector<float> all;
        for (int i = 0; i < S; ++i) { a[i] = d(g); b[i] = d(g); all.push_back(a[i]); all.push_back(b[i]); }
        bitonic_sort_desc<S>(a);
        bitonic_sort_desc<S>(b);
        for (int i = 0; i < S; ++i) c[i] = fmaxf(a[i], b[S - 1 - i]);
        bitonic_merge_desc<S>(c);
        std::sort(all.begin(), all.end(), [](float x, float y) { return x > y; });
        for (int i = 0; i < S; ++i) CHECK(c[i] == all[i]);
    }
}

static void test_slot() {
    std::mt19937 g(7);
    for (int rep = 0; rep < 2000; ++rep) {
        int n = 1 + g() % 40;
        std::vector<int> start(n + 1, 0);
        for (int j = 0; j < n; ++j) start[j + 1] = start[j] + (g() % 3 == 0 ? 0 : int(g() % 5));
        for (int x = 0; x < start[n]; ++x) {
            int j = upper_slot(start.data(), n, x);
            CHECK(j >= 0 && j < n && start[j] <= x && x < start[j + 1]);
        }
    }
}

int main() {
    test_sort8();
    test_insertion<2>(); test_insertion<3>(); test_insertion<4>(); test_insertion<8>(); test_insertion<16>();
    test_sort<1>(); test_sort<2>(); test_sort<4>(); test_sort<8>(); test_sort<16>(); test_sort<32>();
    test_merge<1>(); test_merge<2>(); test_merge<4>(); test_merge<8>(); test_merge<16>();
    test_top<8, 1>(); test_top<8, 2>(); test_top<8, 4>(); test_top<8, 8>();
    test_top<16, 1>(); test_top<16, 2>(); test_top<16, 4>(); test_top<16, 8>(); test_top<16, 16>();
    test_top<32, 1>(); test_top<32, 2>(); test_top<32, 4>(); test_top<32, 8>(); test_top<32, 16>();
    test_pair_fold<1>(); test_pair_fold<2>(); test_pair_fold<4>(); test_pair_fold<8>(); test_pair_fold<16>();
    test_slot();
    if (fails) { std::printf("%d failures\n", fails); return 1; }
    std::printf("ok\n");
    return 0;
}
