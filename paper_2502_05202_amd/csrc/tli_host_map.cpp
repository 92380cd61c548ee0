// tli_host_map.cpp -- Host side of tli_build_map: argument checks, the vocabulary intersection's tables, the host replay of what the
// residual-scan kernel does with them, and the string join that resolves two vocabularies into d2t.  No HIP call
// and no HIP type: this file is also built alone with -fsanitize=address,undefined for the CPU tests.
#include "tli_host_map.h"

#include <algorithm>
#include <cstring>
#include <string_view>
#include <unordered_map>

namespace tli_host {

using namespace tli_layout;

namespace {
inline Int2 mk_i2(int32_t x, int32_t y) { return Int2{x, y}; }
inline UInt2 mk_u2(uint32_t x, uint32_t y) { return UInt2{x, y}; }
}  // namespace

int build_host_map(const int32_t* d2t_host, int32_t Vd, int32_t Vt, HostMap& hm) {
    if (!d2t_host || !vocab_ok(Vd) || !vocab_ok(Vt)) return TLI_ERR_INVALID_ARG;
    const size_t Vd_pad = ((size_t)Vd + 7) & ~(size_t)7, Vt_pad = ((size_t)Vt + 7) & ~(size_t)7;
    std::vector<int32_t>&d2t = hm.d2t, &t2d = hm.t2d, &sh_x = hm.sh_x;
    d2t.assign(Vd_pad, -1);
    t2d.assign(Vt_pad, -1);
    int32_t S = 0;
    for (int32_t x = 0; x < Vd; ++x) {
        const int32_t t = d2t_host[x];
        if (t == -1) continue;
        if (t < 0 || t >= Vt) return TLI_ERR_OUT_OF_RANGE;
        if (t2d[t] != -1) return TLI_ERR_NOT_INJECTIVE;
        t2d[t] = x;
        d2t[x] = t;
        ++S;
    }
    if (S == 0) return TLI_ERR_EMPTY_INTERSECTION;
    hm.S = S;
    // rank -> drafter id, and per dtype the lists of the residual scan (see tli_map)
    sh_x.resize(S);
    {
        int32_t r = 0;
        for (int32_t x = 0; x < Vd; ++x)
            if (d2t[x] >= 0) sh_x[r++] = x;
    }
    HostScan* hs = hm.hs;
    std::vector<uint64_t>* lmask = hm.lmask;
    for (int dt = 0; dt < 2; ++dt) {
        HostScan& h = hs[dt];
        const int CH = dt == TLI_BF16 ? chunk_elems<TLI_BF16>() : chunk_elems<TLI_F32>();
        const int cap = dt == TLI_BF16 ? part_cap<TLI_BF16>() : part_cap<TLI_F32>();
        const int epv = dt == TLI_BF16 ? 8 : 4;
        const uint32_t esz = dt == TLI_BF16 ? 2 : 4;
        const int nC = (Vt + CH - 1) / CH;
        // pairs per chunk, then parts: runs of whole chunks, filled evenly but never beyond what LDS holds
        std::vector<int32_t> cc(nC, 0);
        for (int32_t r = 0; r < S; ++r) ++cc[d2t[sh_x[r]] / CH];
        const int want = (S + cap - 1) / cap;
        const int64_t even = ((int64_t)S + want - 1) / want;
        int32_t biggest = 0;
        for (int c = 0; c < nC; ++c) biggest = cc[c] > biggest ? cc[c] : biggest;
        const int64_t limit = even + biggest < cap ? even + biggest : cap;
        h.cb.assign(1, 0);
        int64_t acc = 0;
        for (int c = 0; c < nC; ++c) {
            if ((acc > 0 && acc + cc[c] > limit) || c - h.cb.back() >= kMaxPartChunks) { h.cb.push_back(c); acc = 0; }
            acc += cc[c];
        }
        h.cb.push_back(nC);
        const int nparts = (int)h.cb.size() - 1;
        std::vector<int32_t> part_of_chunk(nC);
        h.part_n.assign(nparts, 0);
        h.max_part_chunks = 0;
        for (int p = 0; p < nparts; ++p) {
            for (int c = h.cb[p]; c < h.cb[p + 1]; ++c) { part_of_chunk[c] = p; h.part_n[p] += cc[c]; }
            if (h.cb[p + 1] - h.cb[p] > h.max_part_chunks) h.max_part_chunks = h.cb[p + 1] - h.cb[p];
        }
        h.pl_g.assign(nC + 1, 0);
        for (int c = 0; c < nC; ++c) h.pl_g[c + 1] = h.pl_g[c] + (cc[c] + kPairG - 1) / kPairG;
        for (int layout = 0; layout < 2; ++layout) {
            // staging table: what the sweep over a drafter row (element index = drafter id in the full layout,
            // rank in the compact one) keeps of every vector for a part, and where it puts it
            const int64_t elems = layout ? S : Vd;
            const int NV = (int)(((elems + epv - 1) / epv + kWave - 1) / kWave) * kWave;
            h.NV[layout] = NV;
            h.stab[layout].assign((size_t)nparts * NV, 0);
            h.grange[layout].assign(nparts, mk_i2(NV / kWave, 0));
            for (int32_t r = 0; r < S; ++r) {
                const int64_t x = layout ? r : sh_x[r];
                const int p = part_of_chunk[d2t[sh_x[r]] / CH];
                h.stab[layout][(size_t)p * NV + x / epv] |= 1u << (16 + x % epv);
                const int g = (int)(x / epv / kWave);
                if (g < h.grange[layout][p].x) h.grange[layout][p].x = g;
                if (g + 1 > h.grange[layout][p].y) h.grange[layout][p].y = g + 1;
            }
            for (int p = 0; p < nparts; ++p) {
                if (h.grange[layout][p].y == 0) h.grange[layout][p] = mk_i2(0, 0);  // a part without pairs
                uint32_t run = 0;
                for (int vi = 0; vi < NV; ++vi) {
                    uint32_t& w = h.stab[layout][(size_t)p * NV + vi];
                    const uint32_t cnt = (uint32_t)__builtin_popcount(w >> 16);
                    w |= cnt ? run : 0;  // vectors that keep nothing never use the index
                    run += cnt;
                }
            }
            // pairs grouped by target chunk.  A group is read by a wave as two rounds of 64 two-byte (four-byte) LDS
            // reads of the target logits and two of the staged drafter logits; LDS serves a half-wave of 32 lanes
            // from 32 banks of 4 bytes in one pass when no two lanes want different words of one bank.  So a
            // chunk's pairs are dealt to the half-wave slots of its groups (4 per group) one by one, the pairs from
            // the most crowded banks first, each to the slot where it adds the fewest passes (then the fewest
            // lanes of its two banks, then the emptiest).  Any fixed order is as good as any other for the sums.
            const uint32_t dummy = (uint32_t)(dt == TLI_BF16 ? dummy_index<TLI_BF16>() : dummy_index<TLI_F32>()) << kPairShift;
            h.pl_e[layout].assign(((size_t)h.pl_g[nC] + kPairU) * kWave, mk_u2(dummy, dummy));
            std::vector<std::vector<uint32_t>> of_chunk(nC);
            for (int c = 0; c < nC; ++c) of_chunk[c].reserve(cc[c]);
            for (int32_t r = 0; r < S; ++r) {
                const int64_t x = layout ? r : sh_x[r];
                const int32_t t = d2t[sh_x[r]];
                const int c = t / CH, p = part_of_chunk[c];
                const uint32_t w = h.stab[layout][(size_t)p * NV + x / epv];
                const uint32_t pos = (w & 0xffffu) + (uint32_t)__builtin_popcount((w >> 16) & ((1u << (x % epv)) - 1u));
                of_chunk[c].push_back((uint32_t)(t % CH) * esz | (pos << kPairShift));
            }
            constexpr int kBanks = 32, kHalf = kWave / 2;
            std::vector<int32_t> order, degx(kBanks), degy(kBanks);
            std::vector<uint8_t> cx, cy;
            std::vector<int32_t> fill, mx, my;
            for (int c = 0; c < nC; ++c) {
                const std::vector<uint32_t>& es = of_chunk[c];
                const int n = (int)es.size();
                const int H = (h.pl_g[c + 1] - h.pl_g[c]) * (kPairG / kHalf);
                auto bank_x = [&](uint32_t e) { return (int)(((e & 0xffffu) / 4u) % kBanks); };
                auto bank_y = [&](uint32_t e) { return (int)(((e >> kPairShift) * esz / 4u) % kBanks); };
                std::fill(degx.begin(), degx.end(), 0);
                std::fill(degy.begin(), degy.end(), 0);
                for (uint32_t e : es) { ++degx[bank_x(e)]; ++degy[bank_y(e)]; }
                order.resize(n);
                for (int i = 0; i < n; ++i) order[i] = i;
                std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
                    return degx[bank_x(es[a])] + degy[bank_y(es[a])] > degx[bank_x(es[b])] + degy[bank_y(es[b])];
                });
                cx.assign((size_t)H * kBanks, 0);
                cy.assign((size_t)H * kBanks, 0);
                fill.assign(H, 0); mx.assign(H, 1); my.assign(H, 1);
                for (int i : order) {
                    const uint32_t e = es[i];
                    const int bx = bank_x(e), by = bank_y(e);
                    int best = -1;
                    int64_t best_key = 0;
                    for (int s = 0; s < H; ++s) {
                        if (fill[s] >= kHalf) continue;
                        const int nx = cx[(size_t)s * kBanks + bx] + 1, ny = cy[(size_t)s * kBanks + by] + 1;
                        const int added = (nx > mx[s] ? nx - mx[s] : 0) + (ny > my[s] ? ny - my[s] : 0);
                        const int64_t key = ((int64_t)added << 32) | ((int64_t)(nx + ny) << 16) | fill[s];
                        if (best < 0 || key < best_key) { best = s; best_key = key; }
                    }
                    const int s = best;  // n <= 32 * H: a slot with a free lane exists
                    const int nx = ++cx[(size_t)s * kBanks + bx], ny = ++cy[(size_t)s * kBanks + by];
                    if (nx > mx[s]) mx[s] = nx;
                    if (ny > my[s]) my[s] = ny;
                    // slot s = group s / 4, the lanes' first (second) entries for s % 4 < 2 (>= 2), lanes 0..31 or 32..63
                    const int lane = (s % 2) * kHalf + fill[s]++;
                    UInt2& two = h.pl_e[layout][((size_t)h.pl_g[c] + s / 4) * kWave + lane];
                    if ((s % 4) / 2 == 0) two.x = e; else two.y = e;
                }
            }
        }
    }
    // shared-id mask of the drafter vocabulary in lane-mask layout (see mask_bits), padded to whole chunks
    for (int dt = 0; dt < 2; ++dt) {
        const int epv = dt == TLI_BF16 ? 8 : 4;
        const int chunk = kWave * kLoads * epv;
        const size_t nchunks = ((size_t)Vd + chunk - 1) / chunk;
        lmask[dt].assign(nchunks * kLoads * epv, 0);
        for (int32_t x = 0; x < Vd; ++x) {
            if (d2t[x] < 0) continue;
            const int64_t vi = x / epv;
            lmask[dt][(vi >> 6) * epv + (x % epv)] |= 1ull << (vi & 63);
        }
    }
    return TLI_OK;
}

// Replays, on the host, what the residual scan does with the lists of one dtype and one row layout -- the sweep
// that packs a part's drafter logits into LDS, then the walk over every chunk's pair list -- and checks that
// every read stays inside what was built, that every staged slot is written once, and that every shared pair
// (target id, drafter id) is visited exactly once, its two sides matching the map.  0 if so, else the number of
// the first check that failed.
int check_host_scan(const HostMap& hm, int32_t Vd, int32_t Vt, int dt, int layout) {
    const HostScan& h = hm.hs[dt];
    const int CH = dt == TLI_BF16 ? chunk_elems<TLI_BF16>() : chunk_elems<TLI_F32>();
    const int cap = dt == TLI_BF16 ? part_cap<TLI_BF16>() : part_cap<TLI_F32>();
    const uint32_t dummy_idx = (uint32_t)(dt == TLI_BF16 ? dummy_index<TLI_BF16>() : dummy_index<TLI_F32>());
    const int epv = dt == TLI_BF16 ? 8 : 4;
    const uint32_t esz = dt == TLI_BF16 ? 2 : 4;
    const int nC = (Vt + CH - 1) / CH;
    const int nparts = (int)h.part_n.size();
    const int64_t elems = layout ? hm.S : Vd;
    const int64_t nvd = (elems + epv - 1) / epv;
    const int NV = h.NV[layout];
    if ((int)h.cb.size() != nparts + 1 || h.cb[0] != 0 || h.cb[nparts] != nC || (int)h.pl_g.size() != nC + 1) return 1;
    if (NV % kWave != 0 || NV < nvd || h.stab[layout].size() != (size_t)nparts * NV) return 2;
    if (h.pl_e[layout].size() != ((size_t)h.pl_g[nC] + kPairU) * kWave) return 3;
    int64_t total = 0;
    std::vector<std::vector<int64_t>> staged(nparts);
    for (int p = 0; p < nparts; ++p) {
        const int nch = h.cb[p + 1] - h.cb[p];
        if (nch < 1 || nch > kMaxPartChunks || h.part_n[p] < 0 || h.part_n[p] > cap) return 4;
        total += h.part_n[p];
        staged[p].assign(h.part_n[p], -1);
        const Int2 gr = h.grange[layout][p];
        if (gr.x < 0 || gr.y > NV / kWave || (h.part_n[p] > 0 && gr.x >= gr.y)) return 5;
        for (int64_t vi = 0; vi < NV; ++vi) {
            const uint32_t w = h.stab[layout][(size_t)p * NV + vi];
            const bool swept = vi >= (int64_t)gr.x * kWave && vi < (int64_t)gr.y * kWave && vi < nvd;
            if (!swept) {
                if (w >> 16) return 6;  // a logit the sweep never reaches
                continue;
            }
            uint32_t idx = w & 0xffffu;
            for (int i = 0; i < epv; ++i) {
                if (!((w >> (16 + i)) & 1u)) continue;
                const int64_t e = vi * epv + i;
                if (e >= elems || idx >= (uint32_t)h.part_n[p] || staged[p][idx] != -1) return 7;
                staged[p][idx++] = e;
            }
        }
        for (int64_t e : staged[p])
            if (e < 0) return 8;
    }
    if (total != hm.S) return 9;
    std::vector<uint8_t> seen(hm.S, 0);
    std::vector<int32_t> rank_of(Vd, -1);
    for (int32_t r = 0; r < hm.S; ++r) rank_of[hm.sh_x[r]] = r;
    int64_t visited = 0;
    int p = 0;
    for (int c = 0; c < nC; ++c) {
        while (c >= h.cb[p + 1]) ++p;
        if (h.pl_g[c + 1] < h.pl_g[c]) return 10;
        for (int64_t g = h.pl_g[c]; g < h.pl_g[c + 1]; ++g)
            for (int l = 0; l < kWave; ++l) {
                const UInt2 two = h.pl_e[layout][(size_t)g * kWave + l];
                for (uint32_t e : {two.x, two.y}) {
                    const uint32_t toff = e & 0xffffu, idx = e >> kPairShift;
                    if (idx == dummy_idx) {
                        if (toff != 0) return 11;
                        continue;
                    }
                    if (toff % esz || toff / esz >= (uint32_t)CH || idx >= (uint32_t)h.part_n[p]) return 12;
                    const int64_t t = (int64_t)c * CH + toff / esz;
                    const int64_t x = layout ? hm.sh_x[staged[p][idx]] : staged[p][idx];
                    if (t >= Vt || hm.d2t[x] != t) return 13;
                    const int32_t r = rank_of[x];
                    if (seen[r]) return 14;
                    seen[r] = 1;
                    ++visited;
                }
            }
    }
    if (visited != hm.S) return 15;
    for (size_t i = (size_t)h.pl_g[nC] * kWave; i < h.pl_e[layout].size(); ++i) {  // the slack behind the last list
        const UInt2 two = h.pl_e[layout][i];
        if (two.x != dummy_idx << kPairShift || two.y != dummy_idx << kPairShift) return 16;
    }
    return 0;
}

}  // namespace tli_host

extern "C" {

using tli_host::HostMap;
using tli_layout::vocab_ok;

int tli_d2t_from_strings(const char* bytes_d, const int64_t* offs_d, int32_t Vd, const char* bytes_t, const int64_t* offs_t,
                         int32_t Vt, int32_t* d2t_out, int32_t* out_num_shared) {
    if (out_num_shared) *out_num_shared = 0;
    if (!offs_d || !offs_t || !d2t_out || !vocab_ok(Vd) || !vocab_ok(Vt)) return TLI_ERR_INVALID_ARG;
    for (int32_t t = 0; t < Vt; ++t)
        if (offs_t[t] < 0 || offs_t[t + 1] < offs_t[t]) return TLI_ERR_OUT_OF_RANGE;
    for (int32_t x = 0; x < Vd; ++x)
        if (offs_d[x] < 0 || offs_d[x + 1] < offs_d[x]) return TLI_ERR_OUT_OF_RANGE;
    if ((!bytes_t && offs_t[Vt] > 0) || (!bytes_d && offs_d[Vd] > 0)) return TLI_ERR_INVALID_ARG;
    auto token = [](const char* bytes, const int64_t* offs, int32_t i) {
        return std::string_view(bytes ? bytes + offs[i] : "", (size_t)(offs[i + 1] - offs[i]));
    };
    std::unordered_map<std::string_view, int32_t> in_t;
    in_t.reserve((size_t)Vt * 2);
    for (int32_t t = 0; t < Vt; ++t)
        if (!in_t.emplace(token(bytes_t, offs_t, t), t).second) return TLI_ERR_NOT_INJECTIVE;
    std::unordered_map<std::string_view, int32_t> in_d;
    in_d.reserve((size_t)Vd * 2);
    int32_t S = 0;
    for (int32_t x = 0; x < Vd; ++x) {
        const std::string_view s = token(bytes_d, offs_d, x);
        if (!in_d.emplace(s, x).second) return TLI_ERR_NOT_INJECTIVE;
        const auto hit = in_t.find(s);
        d2t_out[x] = hit == in_t.end() ? -1 : hit->second;
        S += hit != in_t.end();
    }
    if (out_num_shared) *out_num_shared = S;
    return TLI_OK;
}

int tli_map_dry_run(const int32_t* d2t_host, int32_t Vd, int32_t Vt, int32_t* out_num_shared, int32_t* out_nparts,
                    int32_t* out_failed_check) {
    if (out_num_shared) *out_num_shared = 0;
    if (out_failed_check) *out_failed_check = 0;
    HostMap hm;
    const int rc = tli_host::build_host_map(d2t_host, Vd, Vt, hm);
    if (rc != TLI_OK) return rc;
    if (out_num_shared) *out_num_shared = hm.S;
    for (int dt = 0; dt < 2; ++dt) {
        if (out_nparts) out_nparts[dt] = (int32_t)hm.hs[dt].part_n.size();
        for (int layout = 0; layout < 2; ++layout) {
            const int bad = tli_host::check_host_scan(hm, Vd, Vt, dt, layout);
            if (bad) {
                if (out_failed_check) *out_failed_check = 1000 * (2 * dt + layout + 1) + bad;
                return TLI_ERR_INTERNAL;
            }
        }
    }
    return TLI_OK;
}


}  // extern "C"
