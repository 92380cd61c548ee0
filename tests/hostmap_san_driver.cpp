// Driver for the sanitizer build of the host-side map builder (tli_host_map.cpp compiled with
// -fsanitize=address,undefined, no HIP): builds seeded vocabulary maps of given shapes, runs tli_map_dry_run (same
// checks and tables as tli_build_map, then the host replay of the residual scan's indexing) and the string join,
// and prints one line per case.  Any sanitizer report makes the process exit non-zero.
//   usage: hostmap_san  Vd Vt S seed mode  [Vd Vt S seed mode ...]
//   mode 0: shared ids at seeded random positions; 1: shared ids bunched at the start of both vocabularies;
//        2: identical vocabularies (S = Vd = Vt, identity); 3: an invalid map (out of range / not injective / empty,
//        by seed % 3); 4: as 0, d2t obtained from token strings by tli_d2t_from_strings
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "tli.h"

static uint64_t g_state;
static uint32_t rnd() {  // splitmix64
    uint64_t z = (g_state += 0x9e3779b97f4a7c15ull);
    z = (z ^ (z >> 30)) * 0xbf58476d1ce4e5b9ull;
    z = (z ^ (z >> 27)) * 0x94d049bb133111ebull;
    return (uint32_t)((z ^ (z >> 31)) >> 16);
}
static std::vector<int32_t> permutation(int32_t n) {
    std::vector<int32_t> p(n);
    for (int32_t i = 0; i < n; ++i) p[i] = i;
    for (int32_t i = n - 1; i > 0; --i) {
        const int32_t j = (int32_t)(rnd() % (uint32_t)(i + 1));
        const int32_t t = p[i]; p[i] = p[j]; p[j] = t;
    }
    return p;
}

int main(int argc, char** argv) {
    int bad = 0;
    for (int a = 1; a + 4 < argc; a += 5) {
        const int32_t Vd = atoi(argv[a]), Vt = atoi(argv[a + 1]);
        int32_t S = atoi(argv[a + 2]);
        const int seed = atoi(argv[a + 3]), mode = atoi(argv[a + 4]);
        g_state = 0x1234567ull + (uint64_t)seed * 7919u;
        std::vector<int32_t> d2t(Vd, -1);
        if (mode == 2) {
            for (int32_t x = 0; x < Vd && x < Vt; ++x) d2t[x] = x;
        } else if (mode == 1) {
            const std::vector<int32_t> pt = permutation(S);
            for (int32_t x = 0; x < S; ++x) d2t[x] = pt[x];
        } else {
            const std::vector<int32_t> pd = permutation(Vd), pt = permutation(Vt);
            for (int32_t i = 0; i < S; ++i) d2t[pd[i]] = pt[i];
        }
        int expect = TLI_OK;
        if (mode == 3) {
            if (seed % 3 == 0) { d2t[0] = Vt; expect = TLI_ERR_OUT_OF_RANGE; }
            else if (seed % 3 == 1) { d2t[0] = 0; d2t[Vd - 1] = 0; expect = TLI_ERR_NOT_INJECTIVE; }
            else { for (auto& v : d2t) v = -1; expect = TLI_ERR_EMPTY_INTERSECTION; }
        }
        if (mode == 4) {  // the same map through token strings: shared tokens get the same string on both sides
            std::vector<std::string> td(Vd), tt(Vt);
            for (int32_t t = 0; t < Vt; ++t) tt[t] = "t" + std::to_string(t);
            for (int32_t x = 0; x < Vd; ++x) td[x] = d2t[x] >= 0 ? tt[d2t[x]] : "d" + std::to_string(x);
            std::string bd, bt;
            std::vector<int64_t> od(Vd + 1, 0), ot(Vt + 1, 0);
            for (int32_t x = 0; x < Vd; ++x) { bd += td[x]; od[x + 1] = (int64_t)bd.size(); }
            for (int32_t t = 0; t < Vt; ++t) { bt += tt[t]; ot[t + 1] = (int64_t)bt.size(); }
            std::vector<int32_t> joined(Vd, -7);
            int32_t Sj = -1;
            const int rcj = tli_d2t_from_strings(bd.data(), od.data(), Vd, bt.data(), ot.data(), Vt, joined.data(), &Sj);
            if (rcj != TLI_OK || joined != d2t) { printf("string join differs (rc %d)\n", rcj); bad = 1; }
            d2t = joined;
        }
        int32_t Sout = -1, nparts[2] = {-1, -1}, failed = -1;
        const int rc = tli_map_dry_run(d2t.data(), Vd, Vt, &Sout, nparts, &failed);
        printf("Vd %d Vt %d S %d seed %d mode %d -> rc %d shared %d nparts %d %d failed_check %d\n", Vd, Vt, S, seed, mode, rc,
               Sout, nparts[0], nparts[1], failed);
        if (rc != expect || (rc == TLI_OK && failed != 0)) bad = 1;
    }
    return bad;
}
