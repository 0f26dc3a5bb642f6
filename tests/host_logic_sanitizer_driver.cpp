// Host logic of the library under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only; no HIP call
// is made): descriptor validation, workspace layout, the planner that splits segments into merged
// dispatches, launch-shape selection and the selector, driven over the benchmark chains and over a few
// thousand random descriptors (most of them invalid: those must be refused, not crash).
#include "../include/pygraph_hip.h"

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

namespace {

struct Rng {
    uint64_t s;
    uint32_t next() { s = s * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(s >> 33); }
    int below(int n) { return (int)(next() % (uint32_t)n); }
};

pg_ref ref(int kind, int index) { return pg_ref{kind, index}; }

pg_kernel_desc kernel(int op, int dtype, int seg, int out, pg_ref a, pg_ref b, pg_ref c, long long n, long long m, long long rows, long long cols,
                      long long inner, float eps) {
    pg_kernel_desc d{};
    d.op = op; d.dtype = dtype; d.segment = seg;
    d.out = ref(PG_REF_INT, out);
    d.in[0] = a; d.in[1] = b; d.in[2] = c;
    d.n = n; d.m = m; d.rows = rows; d.cols = cols; d.inner = inner; d.eps = eps;
    return d;
}
const pg_ref kNone = {PG_REF_NONE, 0};

struct Chain {
    std::vector<pg_kernel_desc> k;
    std::vector<pg_tensor_desc> ext, ints, w;
};

// the decode chain: S sub-blocks of RMSNorm -> GEMV -> GELU -> residual add on [B, H], an input add before some of them
Chain decode(int B, int S, int H, int n_ext, int cut_every) {
    Chain c;
    const int X = 0, T1 = 1, T2 = 2;
    for (int s = 0; s < S; s++) {
        const int seg = cut_every ? s / cut_every : 0;
        for (int j = 1; j < n_ext; j++)
            if ((S * j) / n_ext == s && s > 0)
                c.k.push_back(kernel(PG_ADD, PG_BF16, seg, X, ref(PG_REF_INT, X), ref(PG_REF_EXT, j), kNone, (long long)B * H, (long long)B * H, 1, 0, 0, 0.f));
        const pg_ref x = s == 0 ? ref(PG_REF_EXT, 0) : ref(PG_REF_INT, X);
        c.k.push_back(kernel(PG_RMSNORM, PG_BF16, seg, T1, x, ref(PG_REF_WEIGHT, S + s), kNone, H, 0, B, H, 0, 1e-6f));
        c.k.push_back(kernel(PG_GEMV, PG_BF16, seg, T2, ref(PG_REF_WEIGHT, s), ref(PG_REF_INT, T1), kNone, H, 0, B, H, 0, 0.f));
        c.k.push_back(kernel(PG_GELU, PG_BF16, seg, T2, ref(PG_REF_INT, T2), kNone, kNone, (long long)B * H, 0, 1, 0, 0, 0.f));
        c.k.push_back(kernel(PG_ADD, PG_BF16, seg, X, x, ref(PG_REF_INT, T2), kNone, (long long)B * H, (long long)B * H, 1, 0, 0, 0.f));
    }
    for (int i = 0; i < n_ext; i++) c.ext.push_back(pg_tensor_desc{PG_BF16, 0, (long long)B * H});
    for (int i = 0; i < 3; i++) c.ints.push_back(pg_tensor_desc{PG_BF16, 0, (long long)B * H});
    for (int i = 0; i < S; i++) c.w.push_back(pg_tensor_desc{PG_BF16, 0, (long long)H * H});
    for (int i = 0; i < S; i++) c.w.push_back(pg_tensor_desc{PG_BF16, 0, H});
    return c;
}

// a random chain of decoder-like kernels on [rows, 2048] buffers: valid by construction (operands are read
// only from buffers that earlier kernels wrote in full), then, one time in four, damaged in one place
Chain random_chain(Rng& r) {
    Chain c;
    const int H = 2048;
    const int rows = 1 + (r.below(3) ? r.below(4) : r.below(40));
    const long long N = (long long)rows * H;
    const int n_int = 2 + r.below(5), n_ext = 1 + r.below(3);
    for (int i = 0; i < n_int; i++) c.ints.push_back(pg_tensor_desc{PG_BF16, 0, N * (r.below(8) == 0 ? 2 : 1)});
    for (int i = 0; i < n_ext; i++) c.ext.push_back(pg_tensor_desc{PG_BF16, 0, N});
    c.w.push_back(pg_tensor_desc{PG_BF16, 0, (long long)H * H});   // 0: a weight matrix
    c.w.push_back(pg_tensor_desc{PG_BF16, 0, H});                  // 1: a gain / broadcast vector
    c.w.push_back(pg_tensor_desc{PG_BF16, 0, N});                  // 2: a full-size constant
    std::vector<bool> full(n_int, false);
    auto source = [&]() {                                          // something of N elements that can be read now
        for (int tries = 0; tries < 8; tries++) {
            const int pick = r.below(n_int + n_ext + 1);
            if (pick < n_int) { if (full[pick]) return ref(PG_REF_INT, pick); }
            else if (pick < n_int + n_ext) return ref(PG_REF_EXT, pick - n_int);
            else return ref(PG_REF_WEIGHT, 2);
        }
        return ref(PG_REF_EXT, 0);
    };
    const int nk = 2 + r.below(24);
    int seg = 0;
    for (int i = 0; i < nk; i++) {
        if (i && r.below(9) == 0) seg++;
        const int out = r.below(n_int);
        const int what = r.below(10);
        if (what < 3) {                                            // add / mul, element for element or with a period; sometimes in place
            pg_ref a = source(), b = r.below(3) ? source() : ref(PG_REF_WEIGHT, 1);
            const long long m = b.kind == PG_REF_WEIGHT && b.index == 1 ? (r.below(2) ? H : 5) : N;
            int o = out;
            if (a.kind == PG_REF_INT && r.below(2)) o = a.index;                                   // in place on operand 0
            if (b.kind == PG_REF_INT && b.index == o) b = ref(PG_REF_WEIGHT, 2);                   // never on operand 1
            c.k.push_back(kernel(r.below(2) ? PG_ADD : PG_MUL, PG_BF16, seg, o, a, b, kNone, N, m, 1, 0, 0, 0.f));
            full[o] = true;
        } else if (what < 5) {
            pg_ref a = source();
            const int o = a.kind == PG_REF_INT && r.below(2) ? a.index : out;
            c.k.push_back(kernel(PG_GELU, PG_BF16, seg, o, a, kNone, kNone, N, 0, 1, 0, 0, 0.f));
            full[o] = true;
        } else {                                                   // RMSNorm, often straight into a GEMV, often followed by GELU and a residual add
            pg_ref x = source();
            int t1 = out;
            if (x.kind == PG_REF_INT && x.index == t1) t1 = (t1 + 1) % n_int;
            c.k.push_back(kernel(PG_RMSNORM, PG_BF16, seg, t1, x, ref(PG_REF_WEIGHT, 1), kNone, H, 0, rows, H, 0, 1e-6f));
            full[t1] = true;
            if (r.below(4)) {
                int t2 = r.below(n_int);
                if (t2 == t1) t2 = (t2 + 1) % n_int;
                c.k.push_back(kernel(PG_GEMV, PG_BF16, seg, t2, ref(PG_REF_WEIGHT, 0), ref(PG_REF_INT, t1), kNone, H, 0, rows, H, 0, 0.f));
                full[t2] = true;
                if (r.below(3)) c.k.push_back(kernel(PG_GELU, PG_BF16, seg, t2, ref(PG_REF_INT, t2), kNone, kNone, N, 0, 1, 0, 0, 0.f));
                if (r.below(3) && x.kind == PG_REF_INT && x.index != t2)
                    c.k.push_back(kernel(PG_ADD, PG_BF16, seg, x.index, x, ref(PG_REF_INT, t2), kNone, N, N, 1, 0, 0, 0.f));
            }
        }
    }
    if (r.below(4) == 0) {                                         // damage
        pg_kernel_desc& d = c.k[r.below((int)c.k.size())];
        switch (r.below(8)) {
        case 0: d.out.index = n_int + r.below(3); break;
        case 1: d.in[r.below(2)] = ref(1 + r.below(3), r.below(9)); break;
        case 2: d.n = r.below(2) ? 0 : N + 1; break;
        case 3: d.in[1] = ref(PG_REF_INT, d.out.index); break;
        case 4: d.rows = r.below(2) ? 0 : 1 + r.below(300); break;
        case 5: d.segment += 1 + r.below(3); break;
        case 6: d.op = 6 + r.below(3); break;
        default: d.m = 1 + r.below(5000); break;
        }
    }
    return c;
}

// fp32 elementwise chains of every size class (one element per lane up to 16384 elements, 16-byte vectors above,
// no merging when n is not a whole number of vectors), now and then with an RMSNorm over rows of 1024
Chain random_fp32_chain(Rng& r) {
    Chain c;
    const long long sizes[] = {1, 7, 1024, 4096, 16384, 16385, 16388, 20000, 3 * 1024, 1 << 20};
    const long long N = sizes[r.below(10)];
    const int n_int = 1 + r.below(3);
    for (int i = 0; i < n_int; i++) c.ints.push_back(pg_tensor_desc{PG_F32, 0, N});
    c.ext.push_back(pg_tensor_desc{PG_F32, 0, N});
    c.ext.push_back(pg_tensor_desc{PG_F32, 0, N});
    c.w.push_back(pg_tensor_desc{PG_F32, 0, 1024});
    std::vector<bool> full(n_int, false);
    const int nk = 1 + r.below(20);
    int seg = 0;
    for (int i = 0; i < nk; i++) {
        if (i && r.below(11) == 0) seg++;
        const int out = r.below(n_int);
        int src = r.below(n_int);
        pg_ref a = full[src] ? ref(PG_REF_INT, src) : ref(PG_REF_EXT, r.below(2));
        const int what = r.below(8);
        if (what == 0 && N % 1024 == 0 && !(a.kind == PG_REF_INT && a.index == out)) {
            c.k.push_back(kernel(PG_RMSNORM, PG_F32, seg, out, a, ref(PG_REF_WEIGHT, 0), kNone, 1024, 0, N / 1024, 1024, 0, 1e-5f));
        } else if (what < 3) {
            c.k.push_back(kernel(PG_GELU, PG_F32, seg, out, a, kNone, kNone, N, 0, 1, 0, 0, 0.f));
        } else {
            pg_ref b = r.below(2) ? ref(PG_REF_EXT, r.below(2)) : ref(PG_REF_WEIGHT, 0);
            const long long m = b.kind == PG_REF_WEIGHT ? 1 + r.below(1024) : N;
            c.k.push_back(kernel(r.below(2) ? PG_ADD : PG_MUL, PG_F32, seg, out, a, b, kNone, N, m, 1, 0, 0, 0.f));
        }
        full[out] = true;
    }
    return c;
}

int failures = 0;
#define CHECK(cond) do { if (!(cond)) { std::printf("check failed at line %d: %s\n", __LINE__, #cond); failures++; } } while (0)

// build the chain over made-up device addresses (nothing dereferences them on the host); returns whether it was accepted
bool drive(const Chain& c, bool must_build) {
    size_t need = 0;
    pg_status st = pg_chain_workspace_bytes(c.k.data(), (int32_t)c.k.size(), c.ext.data(), (int32_t)c.ext.size(), c.ints.data(), (int32_t)c.ints.size(), &need);
    if (st != PG_OK) { CHECK(!must_build); CHECK(pg_last_error() && pg_last_error()[0]); return false; }
    std::vector<const void*> wp;
    for (size_t i = 0; i < c.w.size(); i++) wp.push_back(reinterpret_cast<const void*>(0x600000000000ull + i * 0x10000000ull));
    pg_chain* ch = nullptr;
    st = pg_chain_build(c.k.data(), (int32_t)c.k.size(), c.ext.data(), (int32_t)c.ext.size(), c.ints.data(), (int32_t)c.ints.size(), wp.data(), c.w.data(),
                        (int32_t)c.w.size(), reinterpret_cast<void*>(0x700000000000ull), need, &ch);
    if (st != PG_OK) { CHECK(!must_build); CHECK(ch == nullptr); return false; }
    CHECK(ch != nullptr);
    // one byte less must be refused
    pg_chain* small = nullptr;
    CHECK(pg_chain_build(c.k.data(), (int32_t)c.k.size(), c.ext.data(), (int32_t)c.ext.size(), c.ints.data(), (int32_t)c.ints.size(), wp.data(), c.w.data(),
                         (int32_t)c.w.size(), reinterpret_cast<void*>(0x700000000000ull), need - 1, &small) == PG_ENOMEM);
    CHECK(small == nullptr);
    int32_t merged = -1, unmerged = -1;
    CHECK(pg_chain_graph_dispatches(ch, &merged, &unmerged) == PG_OK);
    pg_stats stats{};
    CHECK(pg_chain_stats(ch, &stats) == PG_OK);
    CHECK(unmerged == (int32_t)c.k.size() && merged <= unmerged && merged >= stats.n_segments);
    CHECK((size_t)stats.workspace_bytes == need);
    for (int32_t i = 0; i < (int32_t)c.k.size(); i++) {
        uint32_t wg = 0, th = 0;
        CHECK(pg_chain_launch_shape(ch, i, &wg, &th) == PG_OK && wg >= 1 && th >= 64 && th <= 1024);
    }
    CHECK(pg_set_dispatch_merge(ch, 0) == PG_OK && pg_set_dispatch_merge(ch, 1) == PG_OK);
    pg_chain_destroy(ch);
    return true;
}

}  // namespace

int main() {
    // the benchmark chain at every batch bucket, whole and cut into segments of odd and even length
    for (int B : {1, 2, 3, 4, 5, 8, 16, 17, 32, 64, 128})
        for (int cut : {0, 1, 2, 3, 7}) CHECK(drive(decode(B, 24, 2048, 8, cut), true));
    CHECK(drive(decode(1, 120, 2048, 32, 0), true));
    // a hidden size the merged forms do not serve
    CHECK(drive(decode(2, 6, 1024, 3, 0), true));
    Rng r{20250317ull};
    int built = 0, total = 6000;
    for (int i = 0; i < total; i++) built += drive(random_chain(r), false) ? 1 : 0;
    for (int i = 0; i < 2000; i++) CHECK(drive(random_fp32_chain(r), true));
    std::printf("random descriptors: %d of %d accepted\n", built, total);
    CHECK(built > total / 2 && built < total);
    // the selector: strict '<' scan in mode order
    const double cost[2][3] = {{3.0, 2.0, 2.0}, {1.0, 1.0, 0.5}};
    uint8_t mode[2] = {9, 9};
    CHECK(pg_select(&cost[0][0], 2, mode) == PG_OK && mode[0] == PG_GRAPH_COPY && mode[1] == PG_GRAPH_INDIRECT);
    if (failures) { std::printf("host logic sanitizer driver: %d failures\n", failures); return 1; }
    std::printf("host logic sanitizer driver: ok\n");
    return 0;
}
