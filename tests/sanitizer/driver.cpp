// Drives the host plan code through the C ABI: for every matrix given on the command line
// (rowptr / colidx / vals as raw little-endian files, vals may be missing) it builds
// AG_FLAG_HOST_ONLY plans for several block caps and both community-detection methods, reads the
// export and the statistics, and destroys the plan.  Built with -fsanitize=address,undefined.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "adaptgear.h"

template <class T>
static std::vector<T> read_all(const char *path, bool optional)
{
    std::vector<T> v;
    FILE *f = std::fopen(path, "rb");
    if (!f) {
        if (optional) return v;
        std::perror(path);
        std::exit(2);
    }
    std::fseek(f, 0, SEEK_END);
    const long bytes = std::ftell(f);
    std::fseek(f, 0, SEEK_SET);
    v.resize((size_t)bytes / sizeof(T));
    if (!v.empty() && std::fread(v.data(), sizeof(T), v.size(), f) != v.size()) std::exit(2);
    std::fclose(f);
    return v;
}

int main(int argc, char **argv)
{
    for (int a = 1; a + 2 < argc; a += 3) {
        const auto rp = read_all<int32_t>(argv[a], false);
        const auto ci = read_all<int32_t>(argv[a + 1], false);
        const auto va = read_all<float>(argv[a + 2], true);
        ag_csr A{};
        A.n = (int64_t)rp.size() - 1;
        A.nnz = (int64_t)ci.size();
        A.rowptr = rp.data();
        A.colidx = ci.data();
        A.vals = va.empty() ? nullptr : va.data();
        for (int method = 0; method < 2; ++method)
            for (int cap : {128, 16, 40}) {
                ag_options o{};
                o.block_cap = cap;
                o.method = method;
                o.flags = AG_FLAG_HOST_ONLY;
                ag_plan *p = nullptr;
                const int rc = ag_plan_create(&A, A.n, 32, &o, &p);
                if (rc) { std::printf("create failed %d: %s\n", rc, ag_last_error()); return 1; }
                ag_export e{};
                ag_stats s{};
                if (ag_plan_export(p, &e) || ag_plan_stats(p, &s)) return 1;
                long chk = 0;
                for (int64_t i = 0; i < e.n; ++i) chk += e.perm[i] ^ e.iperm[i];
                for (int64_t i = 0; i < e.nnz_intra; ++i) chk += e.intra_col[i];
                for (int64_t i = 0; i < e.nnz_inter; ++i) chk += e.inter_col[i];
                ag_plan *q = nullptr;
                if (ag_plan_clone_for_width(p, 7, &q)) return 1;
                float y = 0.f;
                if (ag_aggregate(q, &y, &y, nullptr) != AG_ERR_UNSUPPORTED) return 1;   // host-only plans refuse
                ag_plan_destroy(q);
                std::printf("%s method %d cap %d n=%ld blocks=%d dense=%d intra=%ld inter=%ld chk=%ld\n", argv[a], method,
                            cap, (long)e.n, e.n_blocks, s.n_dense_blocks, (long)e.nnz_intra, (long)e.nnz_inter, chk);
                ag_plan_destroy(p);
            }
    }
    return 0;
}
