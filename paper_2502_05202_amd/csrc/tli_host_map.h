// tli_host_map.h -- What tli_build_map computes before it touches a device: the vocabulary intersection's tables as host vectors.
// Plain C++ (no HIP): tli_host_map.cpp also builds on its own, with the address and undefined-behaviour sanitizers,
// for the CPU test of the table builder.
#pragma once

#include <cstdint>
#include <vector>

#include "tli.h"
#include "tli_layout.h"

namespace tli_host {

struct HostScan {  // the residual scan's lists for one dtype (see tli_map::Scan)
    std::vector<int32_t> cb, part_n, pl_g;
    int max_part_chunks = 0;
    int NV[2];
    std::vector<uint32_t> stab[2];
    std::vector<tli_layout::Int2> grange[2];
    std::vector<tli_layout::UInt2> pl_e[2];
};
struct HostMap {
    int32_t S = 0;
    std::vector<int32_t> d2t, t2d, sh_x;
    HostScan hs[2];
    std::vector<uint64_t> lmask[2];
};

// argument checks (TLI_ERR_INVALID_ARG / OUT_OF_RANGE / NOT_INJECTIVE / EMPTY_INTERSECTION) and every table
int build_host_map(const int32_t* d2t_host, int32_t Vd, int32_t Vt, HostMap& hm);
// replay of the residual scan's indexing on the tables of one dtype and layout: 0, or the number of the failed check
int check_host_scan(const HostMap& hm, int32_t Vd, int32_t Vt, int dt, int layout);

}  // namespace tli_host
