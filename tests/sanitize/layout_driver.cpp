// Test driver: the library's host-side layout builder and gather-plan builder (layout.cpp,
// plan.cpp) on a batch read from a binary file; everything they produce is written to another
// file.  Built with -fsanitize=address,undefined by tests/test_sanitizers.py and compared with
// what the ordinary library reports through the C ABI.  Test infrastructure only.
//
// Input: int32 B, e_tot; int32 n_nodes[B], n_edges[B], src[e_tot], dst[e_tot].
// Output: int32 status; then, if 0: int64 n_tot, e_tot; int32 max_depth; int32 td_level[n_tot],
// bu_level[n_tot], td_order[n_tot], bu_order[n_tot]; int64 par_ptr[n_tot + 1], chi_ptr[n_tot + 1];
// int32 par_idx[e_tot], chi_idx[e_tot]; per direction the gather plan of the matrix-core sweep
// kernel: int64 sizes of ck_off / rec / ovf, then the three arrays.
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "internal.h"

namespace pl {
static std::string g_error;
void set_error(const std::string &msg) { g_error = msg; }
int fail(int code, const std::string &msg)
{
    g_error = msg;
    return code;
}
int hip_fail(hipError_t, const char *what) { return fail(PL_ERR_HIP, what); }
}  // namespace pl

template <typename T>
static std::vector<T> take(FILE *f, size_t n)
{
    std::vector<T> v(n);
    if (n && fread(v.data(), sizeof(T), n, f) != n) {
        fprintf(stderr, "short read\n");
        exit(2);
    }
    return v;
}

template <typename T>
static void put(FILE *o, const std::vector<T> &v)
{
    if (!v.empty()) fwrite(v.data(), sizeof(T), v.size(), o);
}

int main(int argc, char **argv)
{
    if (argc != 3) return 2;
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 2;
    const std::vector<int32_t> hd = take<int32_t>(f, 2);
    const int32_t B = hd[0], e_tot = hd[1];
    const auto n_nodes = take<int32_t>(f, B), n_edges = take<int32_t>(f, B);
    const auto src = take<int32_t>(f, e_tot), dst = take<int32_t>(f, e_tot);
    fclose(f);
    pl::HostLayout L;
    const int32_t status = pl::build_layout(B, n_nodes.data(), n_edges.data(), src.data(), dst.data(), &L);
    FILE *o = fopen(argv[2], "wb");
    if (!o) return 2;
    fwrite(&status, sizeof(status), 1, o);
    if (status == 0) {
        fwrite(&L.n_tot, sizeof(int64_t), 1, o);
        fwrite(&L.e_tot, sizeof(int64_t), 1, o);
        fwrite(&L.max_depth, sizeof(int32_t), 1, o);
        put(o, L.td_level);
        put(o, L.bu_level);
        put(o, L.td_order);
        put(o, L.bu_order);
        put(o, L.par_ptr);
        put(o, L.chi_ptr);
        put(o, L.par_idx);
        put(o, L.chi_idx);
        for (int dir = 0; dir < 2; ++dir) {
            pl::SweepPlanHost P;
            const int rc = pl::build_sweep_plan(L, dir, &P);
            if (rc) return 3;
            const int64_t sizes[3] = {static_cast<int64_t>(P.ck_off.size()), static_cast<int64_t>(P.rec.size()),
                                      static_cast<int64_t>(P.ovf.size())};
            fwrite(sizes, sizeof(int64_t), 3, o);
            put(o, P.ck_off);
            put(o, P.rec);
            put(o, P.ovf);
        }
    }
    fclose(o);
    return 0;
}
