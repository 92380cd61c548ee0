// tli_kernels.hip -- gfx950 kernels and C ABI of the TLI draft-and-verify path.
//
// Path (paper: the token-level intersection algorithm + appendix "Standard Speculative Decoding"):
//   draft : q' = softmax over the shared drafter ids (the drafter restricted to T∩D, renormalised),
//           one inverse-CDF sample per row.
//   verify: log-normaliser of each of the K target rows -> accept test per position -> first-reject
//           scan -> extra token from the residual norm(max(0, p - q')) or from the bonus row.
//
// Every kernel here is a streaming scan of logit rows: HBM-bound, no dense contraction, no MFMA.
// A row is cut into chunks of 64 lanes x 4 16-byte loads (2048 bf16 / 1024 fp32 elements); a wave
// owns a chunk, keeps the next chunk's loads in flight while it works on the current one, and
// reduces it to a pair (ref, s) with  sum_{x in chunk} 2^(logit_x * c) = s * 2^ref,  c = log2(e)/temp.
// Chunk pairs are combined in fp64.  Samplers keep the per-chunk pairs, locate the chunk that
// contains u * total and re-read only that chunk.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <type_traits>
#include <vector>

#include "tli.h"
#include "tli_bench.h"
#include "tli_host_map.h"
#include "tli_layout.h"

namespace {

using namespace tli_layout;
using tli_host::HostMap;
using tli_host::HostScan;

#include "tli_device_common.h"
#include "tli_softmax_kernels.h"
#include "tli_verify_kernels.h"
#include "tli_seq_kernels.h"
#include "tli_next_kernels.h"

// ======================================= host side ============================================

struct Plan {
    int nC;      // chunks per row
    int nsplit;  // workgroups per row
    int cps;     // chunks per workgroup
};

Plan make_plan(int V, int rows, int chunk) {
    Plan p;
    p.nC = (V + chunk - 1) / chunk;
#ifndef TLI_TARGET_WGS
#define TLI_TARGET_WGS 2048
#endif
    const int target_wgs = TLI_TARGET_WGS;  // ~8 workgroups of 4 waves on each of the 256 CUs
    int want = (target_wgs + rows - 1) / rows;
    int cap = (p.nC + kWaves - 1) / kWaves;  // keep at least one chunk per wave
    p.nsplit = want < 1 ? 1 : (want > cap ? cap : want);
    p.cps = (p.nC + p.nsplit - 1) / p.nsplit;
    p.nsplit = (p.nC + p.cps - 1) / p.cps;
    return p;
}

// dynamic LDS of k_lse: the chunk pairs a workgroup parks
size_t lse_shmem(const Plan& p) { return (size_t)(p.cps < kLdsChunks ? p.cps : kLdsChunks) * sizeof(float2); }

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Workspace {  // offsets into the caller's scratch
    size_t part, part_d, ws_lse_q, ctab, frow, fbad, tab_ref, tab_s, rmass, total;
};

Workspace layout(int B, int K, int Vt, int Vd, int dtype) {
    const int chunk = dtype == TLI_BF16 ? chunk_elems<TLI_BF16>() : chunk_elems<TLI_F32>();
    const int64_t rows = (int64_t)B * K;
    const Plan pl = make_plan(Vt, (int)rows, chunk);
    const int nCt = (Vt + chunk - 1) / chunk, nCd = (Vd + chunk - 1) / chunk;
    const size_t tab_rows_d = (size_t)rows * nCd, tab_rows_t = (size_t)B * nCt;
    const size_t tab = tab_rows_d > tab_rows_t ? tab_rows_d : tab_rows_t;
    Workspace w;
    size_t off = 0;
    const Plan pd = make_plan(Vd, (int)rows, chunk);
    w.part = off; off += align256((size_t)rows * pl.nsplit * sizeof(Part));
    w.part_d = off; off += align256((size_t)rows * pd.nsplit * sizeof(Part));
    w.ws_lse_q = off; off += align256((size_t)rows * sizeof(double));
    w.ctab = off; off += align256((size_t)rows * nCt * sizeof(float2));
    w.frow = off; off += align256((size_t)B * sizeof(FinalRow));
    w.fbad = off; off += align256((size_t)B * sizeof(int32_t));
    w.tab_ref = off; off += align256(tab * sizeof(float));
    w.tab_s = off; off += align256(tab * sizeof(float));
    // the residual scan's chunk masses, one per chunk of the row the extra token is drawn from
    w.rmass = off; off += align256(tab_rows_t * sizeof(double));
    w.total = off;
    return w;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }


// ---- optional per-kernel timing with HIP events on the caller's stream -------------------------
struct Profile {
    bool on = false;
    uint32_t mask = 0;
    int cap = 0;
    std::vector<hipEvent_t> ev[TLI_KERNEL_COUNT];  // start/stop pairs
    int used[TLI_KERNEL_COUNT] = {};
    int every = 1;                      // record one launch in `every`
    int seen[TLI_KERNEL_COUNT] = {};
} g_prof;

struct KernelTimer {  // records start on construction, stop on destruction, if kernel `id` is being profiled
    int id;
    hipStream_t st;
    bool live;
    KernelTimer(int id_, hipStream_t st_) : id(id_), st(st_), live(false) {
        if (g_prof.on && (g_prof.mask >> id & 1u) && (g_prof.seen[id]++ % g_prof.every) == 0 &&
            g_prof.used[id] + 2 <= (int)g_prof.ev[id].size()) {
            live = true;
            (void)hipEventRecord(g_prof.ev[id][g_prof.used[id]], st);
        }
    }
    ~KernelTimer() {
        if (live) {
            (void)hipEventRecord(g_prof.ev[id][g_prof.used[id] + 1], st);
            g_prof.used[id] += 2;
        }
    }
};

// which form the first steps of tli_verify take: 0 = by batch size, 1 = split (k_lse; the accept tests in the
// residual scan's workgroups), 2 = a workgroup per sequence (k_lse_accept_seq) wherever it fits.  Set by
// tli_tune_final_path (tests and benchmarks).
int g_final_path = 0;

struct DraftOut;
template <int DT, int MASKED>
void launch_draft(const void* logits, int64_t row_stride, int R, int V, float temp, const Plan& pl, float cs,
                  double ratio, const uint64_t* bits, const int32_t* d2t, const DraftOut& o, float* tab_ref,
                  float* tab_s, hipStream_t st);

struct VerifyArgs {
    const tli_map* map;
    const void *logits_t, *logits_d;
    int B, K;
    Plan pl, pf;
    double c_t, c_d, ratio_t, inv_t, inv_d;
    float cs_t;
    const int32_t* tok_d;
    const double* lse_q;
    const float *u_acc, *u_fin;
    int32_t *n_accepted, *out_tok;
    uint8_t* accept;
    double *p_tok, *q_tok, *lse_p;
    int32_t* seq_status;
    Part *part, *part_d;
    double* ws_lse_q;
    Plan pd;
    float cs_d;
    double ratio_d;
    float *tab_ref, *tab_s;
    double* rmass;
    float2* ctab;
    FinalRow* frow;
    int32_t* fbad;
    int union_mode;  // 0: TLI (q' over the shared ids); 1: the union algorithm (q over all of D)
    DrafterView dv;
    int skip_lse_p = 0;  // launch_verify_lse: only the drafter normalisers (if asked for), not the target rows
    int compact;     // drafter rows hold the S shared logits in rank order
    int d_valid;     // valid entries of a drafter row (Vd, or S in the compact layout)
};
template <int DT> void launch_verify(const VerifyArgs& a, hipStream_t st);

}  // namespace

struct tli_map {
    int32_t Vd, Vt, S;
    int device;
    int32_t* d2t;    // dev [Vd padded to 8]
    int32_t* t2d;    // dev [Vt padded to 8]
    uint64_t* lmask[2];  // dev, per dtype: shared-id mask of the drafter vocabulary in lane-mask layout
    int32_t* sh_x;   // dev [S]: drafter id of the shared token of rank r (ranks ascend with the drafter id)
    int32_t* d2r;    // dev [Vd]: rank of a shared drafter id, -1 otherwise   } the index of a token in a drafter row
    int32_t* t2r;    // dev [Vt padded to 8]: rank of a shared target id, -1   } stored in compact (rank-order) layout
    // Per dtype (index = tli_dtype), for the residual scan: the target chunks are cut into nparts parts (runs of
    // whole chunks with at most part_cap shared pairs).  cb [nparts+1] first chunk of a part, part_n [nparts] its
    // pairs.  Per drafter-row layout (0 full, 1 compact): NV vectors in a row (whole groups of 64); stab [nparts][NV]
    // the staging table (which elements of a vector belong to the part, and where they go); grange [nparts] the groups that
    // hold any; pl_e the pairs grouped by target chunk, a chunk's list padded to whole groups of kPairG, entry =
    // byte offset of the target id in its chunk | index of the pair's staged logit << kPairShift (padding entries
    // point at dummy_index; kPairU groups of padding close the list); pl_g [nC+1] first group of every chunk's
    // list (the same for both layouts).
    struct Scan {
        int32_t nparts;
        int32_t max_part_chunks;  // chunks of the largest part
        int32_t* cb;
        int32_t* part_n;
        int32_t* pl_g;
        int32_t NV[2];
        uint32_t* stab[2];
        int2* grange[2];
        uint2* pl_e[2];
    } scan[2];
};

namespace {

ScanLists scan_lists(const tli_map* m, int dt, int layout) {
    const tli_map::Scan& sc = m->scan[dt];
    return ScanLists{sc.nparts, layout ? m->S : m->Vd, sc.NV[layout], sc.cb, sc.part_n, sc.grange[layout],
                     sc.stab[layout], sc.pl_g, sc.pl_e[layout]};
}


template <int DT, int MASKED>
void launch_draft(const void* logits, int64_t row_stride, int R, int V, float temp, const Plan& pl, float cs,
                  double ratio, const uint64_t* bits, const int32_t* d2t, const DraftOut& o, float* tab_ref,
                  float* tab_s, hipStream_t st) {
    if constexpr (!(MASKED & 2)) {
        if (o.thr) {  // rows given with thresholds: the same kernels with the filter compiled in
            launch_draft<DT, MASKED | 2>(logits, row_stride, R, V, temp, pl, cs, ratio, bits, d2t, o, tab_ref, tab_s, st);
            return;
        }
    }
    const double inv_temp = 1.0 / (double)temp;
    if (R <= kRowMaxRows && pl.nC <= kRowChunks) {  // few short rows: each in the registers of one workgroup, one kernel
        KernelTimer t(TLI_KERNEL_DRAFT_SCAN, st);
        hipLaunchKernelGGL((k_draft_row<DT, MASKED>), dim3(R), dim3(kRowWaves * kWave), 0, st, logits, row_stride, V, pl.nC,
                           cs, ratio, inv_temp, bits, d2t, o);
        return;
    }
    if (pl.nsplit == 1 && pl.nC <= kLdsChunks) {  // enough rows to fill the chip with one workgroup per row
        KernelTimer t(TLI_KERNEL_DRAFT_SCAN, st);
        hipLaunchKernelGGL((k_draft_fused<DT, MASKED>), dim3(R), dim3(kWG), 0, st, logits, row_stride, V, pl.nC, cs, ratio,
                           inv_temp, bits, d2t, o);
        return;
    }
    {
        KernelTimer t(TLI_KERNEL_DRAFT_SCAN, st);
        hipLaunchKernelGGL((k_draft_scan<DT, MASKED>), dim3((unsigned)R * pl.nsplit), dim3(kWG), 0, st, logits, row_stride,
                           V, pl.nC, pl.cps, pl.nsplit, cs, ratio, bits, tab_ref, tab_s, o.thr, o.stride);
    }
    {
        KernelTimer t(TLI_KERNEL_DRAFT_PICK, st);
        hipLaunchKernelGGL((k_draft_pick<DT, MASKED>), dim3(R), dim3(kLoads * kWave), 0, st, logits, row_stride, V, pl.nC, cs, ratio,
                           inv_temp, bits, d2t, tab_ref, tab_s, o);
    }
}

// One token per row from softmax(logits / temp), restricted to the shared ids if `bits` is given: argument
// checks, plan, scratch carving and launch shared by the draft entry points and the plain row sampler.
int sample_rows_impl(const void* logits, int dtype, int64_t row_stride, int R, int V, float temp, uint64_t* const* bits2,
                     const int32_t* d2t, const float* u, int32_t* tok, int32_t* tok_t, double* p_tok, double* lse,
                     int32_t* status, int64_t io_stride, void* workspace, size_t workspace_bytes, hipStream_t st,
                     const int32_t* r2d = nullptr, const float* thr = nullptr) {
    if (!logits || !u || !tok || !status || !workspace) return TLI_ERR_INVALID_ARG;
    if (R < 1 || R > 0x7fffffff / 64 || !vocab_ok(V) || !(temp > 0.f) || !std::isfinite(temp) || io_stride < 1)
        return TLI_ERR_INVALID_ARG;
    if (dtype != TLI_F32 && dtype != TLI_BF16) return TLI_ERR_INVALID_ARG;
    const int epv = dtype == TLI_BF16 ? 8 : 4;
    if (row_stride < V || row_stride % epv != 0 || !aligned16(logits) || !aligned16(workspace)) return TLI_ERR_INVALID_ARG;
    const int chunk = dtype == TLI_BF16 ? chunk_elems<TLI_BF16>() : chunk_elems<TLI_F32>();
    Plan pl = make_plan(V, R, chunk);
    // from 4 workgroups per CU on, a row per workgroup (scan and draw in one kernel) beats splitting rows
    if (R >= 1024 && pl.nC <= kLdsChunks) { pl.nsplit = 1; pl.cps = pl.nC; }
    const size_t tab_bytes = align256((size_t)R * pl.nC * sizeof(float));
    if (workspace_bytes < 2 * tab_bytes) return TLI_ERR_ALLOC;
    float* tab_ref = reinterpret_cast<float*>(workspace);
    float* tab_s = reinterpret_cast<float*>(static_cast<char*>(workspace) + tab_bytes);
    const double c_true = kLog2e / (double)temp;
    const float cs = (float)c_true;
    const double ratio = c_true / (double)cs;
    DraftOut o;
    o.u_draft = u; o.tok_d = tok; o.tok_t = tok_t; o.q_tok = p_tok; o.lse_q = lse; o.row_status = status;
    o.stride = io_stride;
    o.r2d = r2d;
    o.thr = thr;
    if (bits2) {
        if (dtype == TLI_BF16)
            launch_draft<TLI_BF16, true>(logits, row_stride, R, V, temp, pl, cs, ratio, bits2[TLI_BF16], d2t, o, tab_ref, tab_s, st);
        else
            launch_draft<TLI_F32, true>(logits, row_stride, R, V, temp, pl, cs, ratio, bits2[TLI_F32], d2t, o, tab_ref, tab_s, st);
    } else {
        if (dtype == TLI_BF16)
            launch_draft<TLI_BF16, false>(logits, row_stride, R, V, temp, pl, cs, ratio, nullptr, d2t, o, tab_ref, tab_s, st);
        else
            launch_draft<TLI_F32, false>(logits, row_stride, R, V, temp, pl, cs, ratio, nullptr, d2t, o, tab_ref, tab_s, st);
    }
    return hipGetLastError() == hipSuccess ? TLI_OK : TLI_ERR_HIP;
}

// argmax of R rows (temperature zero); `bits2` restricts the competition to the shared ids.
int argmax_rows_impl(const void* logits, int dtype, int64_t row_stride, int R, int V, uint64_t* const* bits2,
                     const int32_t* d2t, int32_t* tok, int32_t* tok_t, double* p_tok, double* lse, int32_t* status,
                     int64_t io_stride, void* workspace, size_t workspace_bytes, hipStream_t st) {
    if (!logits || !tok || !status || !workspace) return TLI_ERR_INVALID_ARG;
    if (R < 1 || R > 0x7fffffff / 64 || !vocab_ok(V) || io_stride < 1) return TLI_ERR_INVALID_ARG;
    if (dtype != TLI_F32 && dtype != TLI_BF16) return TLI_ERR_INVALID_ARG;
    const int epv = dtype == TLI_BF16 ? 8 : 4;
    if (row_stride < V || row_stride % epv != 0 || !aligned16(logits) || !aligned16(workspace)) return TLI_ERR_INVALID_ARG;
    const int chunk = dtype == TLI_BF16 ? chunk_elems<TLI_BF16>() : chunk_elems<TLI_F32>();
    const Plan pl = make_plan(V, R, chunk);
    if (workspace_bytes < (size_t)R * pl.nsplit * sizeof(ArgPart)) return TLI_ERR_ALLOC;
    ArgPart* part = reinterpret_cast<ArgPart*>(workspace);
    const dim3 grid((unsigned)R * pl.nsplit);
    {
        KernelTimer t(TLI_KERNEL_DRAFT_SCAN, st);
        if (bits2) {
            if (dtype == TLI_BF16)
                hipLaunchKernelGGL((k_argmax<TLI_BF16, true>), grid, dim3(kWG), 0, st, logits, row_stride, V, pl.nC, pl.cps,
                                   pl.nsplit, bits2[TLI_BF16], part);
            else
                hipLaunchKernelGGL((k_argmax<TLI_F32, true>), grid, dim3(kWG), 0, st, logits, row_stride, V, pl.nC, pl.cps,
                                   pl.nsplit, bits2[TLI_F32], part);
        } else {
            if (dtype == TLI_BF16)
                hipLaunchKernelGGL((k_argmax<TLI_BF16, false>), grid, dim3(kWG), 0, st, logits, row_stride, V, pl.nC, pl.cps,
                                   pl.nsplit, (const uint64_t*)nullptr, part);
            else
                hipLaunchKernelGGL((k_argmax<TLI_F32, false>), grid, dim3(kWG), 0, st, logits, row_stride, V, pl.nC, pl.cps,
                                   pl.nsplit, (const uint64_t*)nullptr, part);
        }
    }
    {
        KernelTimer t(TLI_KERNEL_DRAFT_PICK, st);
        hipLaunchKernelGGL(k_argmax_finish, dim3((R + kWG - 1) / kWG), dim3(kWG), 0, st, part, R, pl.nsplit, d2t, tok, tok_t,
                           p_tok, lse, status, io_stride);
    }
    return hipGetLastError() == hipSuccess ? TLI_OK : TLI_ERR_HIP;
}

// scratch of the row sampler / argmax for R rows of V entries
size_t rows_workspace(int R, int V, int dtype) {
    const int chunk = dtype == TLI_BF16 ? chunk_elems<TLI_BF16>() : chunk_elems<TLI_F32>();
    const Plan pl = make_plan(V, R, chunk);
    const size_t tabs = 2 * align256((size_t)R * pl.nC * sizeof(float));
    const size_t parts = align256((size_t)R * pl.nsplit * sizeof(ArgPart));
    return tabs > parts ? tabs : parts;
}

// drafter normalisers if the caller passed none, then the normaliser partials of the K target rows of every sequence
template <int DT> const double* launch_verify_lse(const VerifyArgs& a, hipStream_t st) {
    const int Vt = a.map->Vt, Vd = a.map->Vd, B = a.B, K = a.K, rows = B * K;
    const double* lse_q = a.lse_q;
    if (!lse_q) {  // the caller did not keep the drafter normalisers: one scan of the drafter rows (masked for TLI
                   // in the full layout; a compact row holds the shared ids only)
        const int64_t rs = a.dv.row_stride;
        if (a.union_mode || a.compact)
            hipLaunchKernelGGL((k_lse<DT, false>), dim3((unsigned)rows * a.pd.nsplit), dim3(kWG), lse_shmem(a.pd), st, a.dv.base, K,
                               (int64_t)K * rs, rs, a.d_valid, a.pd.nC, a.pd.cps, a.pd.nsplit, a.cs_d, a.ratio_d,
                               (const uint64_t*)nullptr, a.part_d, (float2*)nullptr);
        else
            hipLaunchKernelGGL((k_lse<DT, true>), dim3((unsigned)rows * a.pd.nsplit), dim3(kWG), lse_shmem(a.pd), st, a.dv.base, K,
                               (int64_t)K * rs, rs, a.d_valid, a.pd.nC, a.pd.cps, a.pd.nsplit, a.cs_d, a.ratio_d,
                               a.map->lmask[DT], a.part_d, (float2*)nullptr);
        hipLaunchKernelGGL(k_lse_finish, dim3((rows + kWG - 1) / kWG), dim3(kWG), 0, st, a.part_d, rows, a.pd.nsplit,
                           a.ratio_d, a.ws_lse_q);
        lse_q = a.ws_lse_q;
    }
    if (!a.skip_lse_p) {
        KernelTimer t(TLI_KERNEL_LSE, st);
        hipLaunchKernelGGL((k_lse<DT, false>), dim3((unsigned)rows * a.pl.nsplit), dim3(kWG), lse_shmem(a.pl), st, a.logits_t, K,
                           (int64_t)(K + 1) * Vt, (int64_t)Vt, Vt, a.pl.nC, a.pl.cps, a.pl.nsplit, a.cs_t, a.ratio_t,
                           nullptr, a.part, a.ctab, a.fbad);
    }
    return lse_q;
}

// accept tests, first-reject scan and the extra token of every sequence, from the normaliser partials
template <int DT>
void launch_verify_tail(const VerifyArgs& a, const double* lse_q, hipStream_t st, bool accept_done = false) {
    const int Vt = a.map->Vt, Vd = a.map->Vd, B = a.B, K = a.K;
    FinalOut fo;
    fo.u_fin = a.u_fin; fo.n_accepted = a.n_accepted; fo.out_tok = a.out_tok; fo.lse_p = a.lse_p;
    fo.seq_status = a.seq_status;
    AcceptIn in;
    in.part = a.part; in.nsplit = a.pl.nsplit; in.ratio_t = a.ratio_t; in.inv_temp_t = a.inv_t; in.inv_temp_d = a.inv_d;
    in.c_t = a.c_t; in.c_d = a.c_d; in.d2t = a.map->d2t; in.tok_d = a.tok_d; in.lse_q = lse_q; in.u_acc = a.u_acc;
    in.union_mode = a.union_mode;
    AcceptOut out;
    out.n_accepted = a.n_accepted; out.out_tok = a.out_tok; out.accept = a.accept; out.p_tok = a.p_tok;
    out.q_tok = a.q_tok; out.lse_p = a.lse_p; out.seq_status = a.seq_status; out.frow = a.frow;
    // split form: the accept tests run inside the residual scan's workgroups (1.5-3 us less than a kernel of their own:
    // 24.0 -> 22.5 us for one sequence, 44.4 -> 42.8 us for 64, 115.3 -> 113.5 us for 128, same-run A/B)
    const bool fuse = !accept_done;
    const int nparts = a.map->scan[DT].nparts;
    const ScanLists ls = scan_lists(a.map, DT, a.compact ? 1 : 0);
    {
        KernelTimer t(TLI_KERNEL_FINAL_SCAN, st);
        // few sequences: deal the chunks of a (sequence, part) to several workgroups, up to one per CU
        int nsplit = 256 / (B * nparts);
        nsplit = nsplit < 1 ? 1 : (nsplit > 4 ? 4 : nsplit);
        const dim3 grid((unsigned)((B + 7) / 8) * 8 * nparts * nsplit);
        if (fuse)
            hipLaunchKernelGGL((k_final_scan<DT, 0, true>), grid, dim3(kScanWG), 0, st, a.logits_t, a.dv, B, K, Vt, Vd,
                               a.pf.nC, nsplit, ls, a.cs_t, a.ratio_t, a.frow, a.tab_ref, a.tab_s, (double*)nullptr,
                               (double*)nullptr, a.fbad, (const int32_t*)nullptr, a.ctab, a.rmass, in, out);
        else
            hipLaunchKernelGGL((k_final_scan<DT, 0, false>), grid, dim3(kScanWG), 0, st, a.logits_t, a.dv, B, K, Vt, Vd,
                               a.pf.nC, nsplit, ls, a.cs_t, a.ratio_t, a.frow, a.tab_ref, a.tab_s, (double*)nullptr,
                               (double*)nullptr, a.fbad, (const int32_t*)nullptr, a.ctab, a.rmass, AcceptIn(), AcceptOut());
    }
    {
        KernelTimer t(TLI_KERNEL_FINAL_PICK, st);
        hipLaunchKernelGGL(k_final_pick<DT>, dim3(B), dim3(kLoads * kWave), 0, st, a.logits_t, a.dv, K, Vt, Vd, a.pf.nC,
                           a.cs_t, a.ratio_t, a.frow, a.dv.t2x, a.tab_ref, a.tab_s, a.ctab, a.rmass, a.fbad, fo);
    }
}


// A workgroup per sequence runs normalisers and accept tests in one kernel (k_lse_accept_seq) when the batch gives
// every compute unit about one sequence or several (a last round of few workgroups would leave the chip idle) and two
// tables of a row's chunk pairs fit its LDS.
bool use_seq_form(const VerifyArgs& a) {
    if (a.pf.nC > kSeqMaxChunks || g_final_path == 1) return false;
    if (g_final_path == 2) return true;
    const int cus = 256, rounds = (a.B + cus - 1) / cus;
    return a.B >= 200 && (double)a.B / ((double)rounds * cus) >= 0.78;
}

template <int DT> void launch_verify(const VerifyArgs& a, hipStream_t st) {
    if (use_seq_form(a)) {
        VerifyArgs q = a;  // of the first step only the drafter normalisers, if the caller passed none
        q.skip_lse_p = 1;
        const double* lse_q = launch_verify_lse<DT>(q, st);
        SeqIn in;
        in.d2t = a.map->d2t; in.tok_d = a.tok_d; in.lse_q = lse_q; in.u_acc = a.u_acc; in.ratio_t = a.ratio_t;
        in.inv_temp_t = a.inv_t; in.inv_temp_d = a.inv_d; in.c_t = a.c_t; in.c_d = a.c_d; in.cs_t = a.cs_t;
        in.union_mode = a.union_mode;
        SeqOut out;
        out.n_accepted = a.n_accepted; out.out_tok = a.out_tok; out.accept = a.accept; out.p_tok = a.p_tok;
        out.q_tok = a.q_tok; out.lse_p = a.lse_p; out.seq_status = a.seq_status; out.frow = a.frow; out.fbad = a.fbad;
        {
            KernelTimer t(TLI_KERNEL_LSE, st);
            hipLaunchKernelGGL(k_lse_accept_seq<DT>, dim3(a.B), dim3(kSeqWG), 0, st, a.logits_t, a.dv, a.K, a.map->Vt,
                               a.map->Vd, a.pf.nC, in, a.ctab, out);
        }
        launch_verify_tail<DT>(a, lse_q, st, /*accept_done=*/true);
        return;
    }
    const double* lse_q = launch_verify_lse<DT>(a, st);
    launch_verify_tail<DT>(a, lse_q, st);
}

}  // namespace

namespace {
struct DiagLayout { size_t part_t, part_q1, part_q2, frow, fbad, redo, mn, mn2, total; };
DiagLayout diag_layout(const tli_map* map, int B, int K, int dtype) {
    const int chunk = dtype == TLI_BF16 ? chunk_elems<TLI_BF16>() : chunk_elems<TLI_F32>();
    const int rows = B * K;
    const Plan pt = make_plan(map->Vt, rows, chunk), pd = make_plan(map->Vd, rows, chunk);
    DiagLayout w;
    size_t off = 0;
    w.part_t = off; off += align256((size_t)rows * pt.nsplit * sizeof(Part));
    w.part_q1 = off; off += align256((size_t)rows * pd.nsplit * sizeof(Part));
    w.part_q2 = off; off += align256((size_t)rows * pd.nsplit * sizeof(Part));
    w.frow = off; off += align256((size_t)rows * sizeof(FinalRow));
    w.fbad = off; off += align256((size_t)rows * sizeof(int32_t));
    w.redo = off; off += align256((size_t)rows * sizeof(int32_t));
    const size_t tab = (size_t)rows * pt.nC * sizeof(double);
    w.mn = off; off += align256(tab);
    w.mn2 = off; off += align256(tab);
    w.total = off;
    return w;
}

template <int DT>
void launch_diag(const tli_map* map, const void* logits_t, const void* logits_d, int B, int K, float temp_t, float temp_d,
                 double* alpha_tli, double* alpha_union, int32_t* status, char* ws, const DiagLayout& w, hipStream_t st) {
    const int Vt = map->Vt, Vd = map->Vd, rows = B * K;
    const int chunk = chunk_elems<DT>();
    const Plan pt = make_plan(Vt, rows, chunk), pd = make_plan(Vd, rows, chunk);
    const double c_t = kLog2e / (double)temp_t, c_d = kLog2e / (double)temp_d;
    const float cs_t = (float)c_t, cs_d = (float)c_d;
    const double ratio_t = c_t / (double)cs_t, ratio_d = c_d / (double)cs_d;
    Part* part_t = reinterpret_cast<Part*>(ws + w.part_t);
    Part* part_q1 = reinterpret_cast<Part*>(ws + w.part_q1);
    Part* part_q2 = reinterpret_cast<Part*>(ws + w.part_q2);
    FinalRow* frow = reinterpret_cast<FinalRow*>(ws + w.frow);
    int32_t* fbad = reinterpret_cast<int32_t*>(ws + w.fbad);
    double* mn = reinterpret_cast<double*>(ws + w.mn);
    double* mn2 = reinterpret_cast<double*>(ws + w.mn2);
    hipLaunchKernelGGL((k_lse<DT, false>), dim3((unsigned)rows * pt.nsplit), dim3(kWG), lse_shmem(pt), st, logits_t, K,
                       (int64_t)(K + 1) * Vt, (int64_t)Vt, Vt, pt.nC, pt.cps, pt.nsplit, cs_t, ratio_t,
                       (const uint64_t*)nullptr, part_t, (float2*)nullptr);
    hipLaunchKernelGGL((k_lse_both<DT>), dim3((unsigned)rows * pd.nsplit), dim3(kWG), 0, st, logits_d, K, (int64_t)K * Vd,
                       (int64_t)Vd, Vd, pd.nC, pd.cps, pd.nsplit, cs_d, ratio_d, map->lmask[DT], part_q1, part_q2);
    hipLaunchKernelGGL(k_diag_rows, dim3((rows + kWG - 1) / kWG), dim3(kWG), 0, st, part_t, pt.nsplit, part_q1, part_q2,
                       pd.nsplit, rows, K, ratio_t, ratio_d, c_t, c_d, frow, fbad, status);
    const int nparts = map->scan[DT].nparts;
    int nsplit = 256 / (rows * nparts);
    nsplit = nsplit < 1 ? 1 : (nsplit > 4 ? 4 : nsplit);
    const ScanLists ls = scan_lists(map, DT, 0);
    int32_t* redo = reinterpret_cast<int32_t*>(ws + w.redo);
    const dim3 scan_grid((unsigned)((rows + 7) / 8) * 8 * nparts * nsplit);
    const DrafterView dvw{logits_d, (int64_t)Vd, nullptr, map->t2d};
    hipLaunchKernelGGL((k_final_scan<DT, 1>), scan_grid, dim3(kScanWG), 0, st, logits_t, dvw, rows, K, Vt, Vd, pt.nC, nsplit,
                       ls, cs_t, ratio_t, frow, (float*)nullptr, (float*)nullptr, mn, mn2, fbad, (const int32_t*)nullptr,
                       (const float2*)nullptr, (double*)nullptr);
    hipLaunchKernelGGL(k_diag_finish, dim3(rows), dim3(kWave), 0, st, frow, mn, mn2, rows, pt.nC, alpha_tli, alpha_union,
                       redo, 0);
    // the positions whose rates are tiny (normally none: their workgroups leave at once) again, with fp64 arguments
    hipLaunchKernelGGL((k_final_scan<DT, 2>), scan_grid, dim3(kScanWG), 0, st, logits_t, dvw, rows, K, Vt, Vd, pt.nC, nsplit,
                       ls, cs_t, ratio_t, frow, (float*)nullptr, (float*)nullptr, mn, mn2, fbad, redo, (const float2*)nullptr,
                       (double*)nullptr);
    hipLaunchKernelGGL(k_diag_finish, dim3(rows), dim3(kWave), 0, st, frow, mn, mn2, rows, pt.nC, alpha_tli, alpha_union,
                       redo, 1);
}
}  // namespace

// ---- scratch of the entry point that allocates nothing (tli_verify_static) -----------------------------
// A fixed device array that lives in the library's code object: every GPU the library runs on holds its own copy
// at its own address until the process ends.  In host code the array's NAME is only a handle for the symbol, not a
// device address; the address on a given device is asked for once, with that device current, and kept.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// device address of `scratch` on the CURRENT device (which must be `dev`); resolved on first use
int static_scratch(int dev, void** out) {
    if (dev < 0 || dev >= kMaxDevices) return TLI_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return TLI_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return TLI_OK;
}
}  // namespace

extern "C" {

int tli_calib_copy(const void* src, void* dst, size_t bytes, void* hip_stream) {
    if (!src || !dst || bytes == 0 || bytes % 16 != 0 || !aligned16(src) || !aligned16(dst)) return TLI_ERR_INVALID_ARG;
    hipLaunchKernelGGL(k_calib_copy, dim3(4096), dim3(kWG), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const u4v*>(src), static_cast<u4v*>(dst), bytes / 16);
    return hipGetLastError() == hipSuccess ? TLI_OK : TLI_ERR_HIP;
}

int tli_calib_read(const void* src, size_t bytes, size_t slab_bytes, int32_t nontemporal, uint32_t* out, void* hip_stream) {
    constexpr size_t chunk_bytes = (size_t)kWave * kLoads * 16;
    if (!src || !out || !aligned16(src) || slab_bytes == 0 || slab_bytes % chunk_bytes != 0 || bytes == 0 ||
        bytes % slab_bytes != 0 || bytes / slab_bytes > 0x7fffffffu)
        return TLI_ERR_INVALID_ARG;
    const dim3 grid((unsigned)(bytes / slab_bytes));
    const hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (nontemporal)
        hipLaunchKernelGGL(k_calib_read<true>, grid, dim3(kWG), 0, st, static_cast<const u4v*>(src), slab_bytes / 16, out);
    else
        hipLaunchKernelGGL(k_calib_read<false>, grid, dim3(kWG), 0, st, static_cast<const u4v*>(src), slab_bytes / 16, out);
    return hipGetLastError() == hipSuccess ? TLI_OK : TLI_ERR_HIP;
}

int tli_device_info(int32_t* out) {
    if (!out) return TLI_ERR_INVALID_ARG;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return TLI_ERR_HIP;
    const hipDeviceAttribute_t attr[4] = {hipDeviceAttributeMemoryClockRate, hipDeviceAttributeMemoryBusWidth,
                                          hipDeviceAttributeMultiprocessorCount, hipDeviceAttributeClockRate};
    for (int i = 0; i < 4; ++i) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, attr[i], dev) != hipSuccess) v = 0;
        out[i] = v;
    }
    (void)hipGetLastError();  // an attribute the runtime does not know is reported as 0, not as a sticky error
    return TLI_OK;
}

int tli_profile_enable(uint32_t kernel_mask, int32_t max_calls, int32_t every) {
    tli_profile_disable();
    if (max_calls < 1 || max_calls > (1 << 20) || every < 1) return TLI_ERR_INVALID_ARG;
    for (int k = 0; k < TLI_KERNEL_COUNT; ++k) {
        if (!(kernel_mask >> k & 1u)) continue;
        g_prof.ev[k].resize((size_t)2 * max_calls);
        for (auto& e : g_prof.ev[k])
            if (hipEventCreate(&e) != hipSuccess) { tli_profile_disable(); return TLI_ERR_HIP; }
    }
    g_prof.mask = kernel_mask;
    g_prof.cap = max_calls;
    g_prof.every = every;
    g_prof.on = true;
    return TLI_OK;
}

int tli_profile_collect(int32_t kernel, double* total_ms, int32_t* launches) {
    if (kernel < 0 || kernel >= TLI_KERNEL_COUNT || !total_ms || !launches) return TLI_ERR_INVALID_ARG;
    double tot = 0.0;
    const int n = g_prof.used[kernel];
    for (int i = 0; i + 1 < n; i += 2) {
        if (hipEventSynchronize(g_prof.ev[kernel][i + 1]) != hipSuccess) return TLI_ERR_HIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_prof.ev[kernel][i], g_prof.ev[kernel][i + 1]) != hipSuccess) return TLI_ERR_HIP;
        tot += ms;
    }
    *total_ms = tot;
    *launches = n / 2;
    g_prof.used[kernel] = 0;
    return TLI_OK;
}

int tli_tune_final_path(int32_t path) {
    if (path < 0 || path > 2) return TLI_ERR_INVALID_ARG;
    g_final_path = path;
    return TLI_OK;
}

void tli_profile_disable(void) {
    for (int k = 0; k < TLI_KERNEL_COUNT; ++k) {
        for (auto& e : g_prof.ev[k])
            if (e) (void)hipEventDestroy(e);
        g_prof.ev[k].clear();
        g_prof.used[k] = 0;
        g_prof.seen[k] = 0;
    }
    g_prof.on = false;
    g_prof.mask = 0;
}


const char* tli_status_string(int status) {
    switch (status) {
        case TLI_OK: return "TLI_OK";
        case TLI_ERR_INVALID_ARG: return "TLI_ERR_INVALID_ARG";
        case TLI_ERR_OUT_OF_RANGE: return "TLI_ERR_OUT_OF_RANGE";
        case TLI_ERR_NOT_INJECTIVE: return "TLI_ERR_NOT_INJECTIVE";
        case TLI_ERR_EMPTY_INTERSECTION: return "TLI_ERR_EMPTY_INTERSECTION";
        case TLI_ERR_ALLOC: return "TLI_ERR_ALLOC";
        case TLI_ERR_HIP: return "TLI_ERR_HIP";
        case TLI_ERR_INTERNAL: return "TLI_ERR_INTERNAL";
        case TLI_ERR_TOO_LARGE: return "TLI_ERR_TOO_LARGE";
        default: return "TLI_ERR_UNKNOWN";
    }
}

int tli_build_map(const int32_t* d2t_host, int32_t Vd, int32_t Vt, tli_map** out_map, int32_t* out_num_shared) {
    if (out_map) *out_map = nullptr;
    if (out_num_shared) *out_num_shared = 0;
    if (!out_map) return TLI_ERR_INVALID_ARG;
    HostMap hm;
    const int rc = tli_host::build_host_map(d2t_host, Vd, Vt, hm);
    if (rc != TLI_OK) return rc;
    const int32_t S = hm.S;
    const std::vector<int32_t>&d2t = hm.d2t, &t2d = hm.t2d, &sh_x = hm.sh_x;
    const HostScan* hs = hm.hs;
    const std::vector<uint64_t>* lmask = hm.lmask;
    const size_t Vd_pad = d2t.size(), Vt_pad = t2d.size();
    tli_map* m = new (std::nothrow) tli_map();
    if (!m) return TLI_ERR_ALLOC;
    m->Vd = Vd; m->Vt = Vt; m->S = S; m->d2t = nullptr; m->t2d = nullptr; m->lmask[0] = m->lmask[1] = nullptr;
    m->sh_x = nullptr; m->d2r = nullptr; m->t2r = nullptr;
    for (int dt = 0; dt < 2; ++dt) {
        tli_map::Scan& sc = m->scan[dt];
        sc.nparts = (int32_t)hs[dt].part_n.size();
        sc.max_part_chunks = hs[dt].max_part_chunks;
        sc.cb = sc.part_n = sc.pl_g = nullptr;
        for (int layout = 0; layout < 2; ++layout) {
            sc.NV[layout] = hs[dt].NV[layout];
            sc.stab[layout] = nullptr; sc.grange[layout] = nullptr; sc.pl_e[layout] = nullptr;
        }
    }
    if (hipGetDevice(&m->device) != hipSuccess) { delete m; return TLI_ERR_HIP; }
    {   // the static scratch of tli_verify_static is looked up here, so that call itself only enqueues kernels
        void* unused = nullptr;
        (void)static_scratch(m->device, &unused);
    }
    bool ok = hipMalloc(&m->d2t, d2t.size() * 4) == hipSuccess && hipMalloc(&m->t2d, t2d.size() * 4) == hipSuccess &&
              hipMalloc(&m->lmask[0], lmask[0].size() * 8) == hipSuccess &&
              hipMalloc(&m->lmask[1], lmask[1].size() * 8) == hipSuccess;
    if (!ok) { tli_free_map(m); return TLI_ERR_ALLOC; }
    ok = hipMemcpy(m->d2t, d2t.data(), d2t.size() * 4, hipMemcpyHostToDevice) == hipSuccess &&
         hipMemcpy(m->t2d, t2d.data(), t2d.size() * 4, hipMemcpyHostToDevice) == hipSuccess &&
         hipMemcpy(m->lmask[0], lmask[0].data(), lmask[0].size() * 8, hipMemcpyHostToDevice) == hipSuccess &&
         hipMemcpy(m->lmask[1], lmask[1].data(), lmask[1].size() * 8, hipMemcpyHostToDevice) == hipSuccess;
    if (!ok) { tli_free_map(m); return TLI_ERR_HIP; }
    std::vector<int32_t> d2r(Vd_pad, -1), t2r(Vt_pad, -1);
    for (int32_t r = 0; r < S; ++r) { d2r[sh_x[r]] = r; t2r[d2t[sh_x[r]]] = r; }
    if (hipMalloc(&m->sh_x, (size_t)S * 4) != hipSuccess || hipMalloc(&m->d2r, d2r.size() * 4) != hipSuccess ||
        hipMalloc(&m->t2r, t2r.size() * 4) != hipSuccess) {
        tli_free_map(m);
        return TLI_ERR_ALLOC;
    }
    if (hipMemcpy(m->sh_x, sh_x.data(), (size_t)S * 4, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(m->d2r, d2r.data(), d2r.size() * 4, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(m->t2r, t2r.data(), t2r.size() * 4, hipMemcpyHostToDevice) != hipSuccess) {
        tli_free_map(m);
        return TLI_ERR_HIP;
    }
    for (int dt = 0; dt < 2; ++dt) {
        tli_map::Scan& sc = m->scan[dt];
        const HostScan& h = hs[dt];
        const struct { void** dev; const void* host; size_t bytes; } lists[] = {
            {(void**)&sc.cb, h.cb.data(), h.cb.size() * 4},
            {(void**)&sc.part_n, h.part_n.data(), h.part_n.size() * 4},
            {(void**)&sc.pl_g, h.pl_g.data(), h.pl_g.size() * 4},
            {(void**)&sc.stab[0], h.stab[0].data(), h.stab[0].size() * 4},
            {(void**)&sc.stab[1], h.stab[1].data(), h.stab[1].size() * 4},
            {(void**)&sc.grange[0], h.grange[0].data(), h.grange[0].size() * sizeof(Int2)},
            {(void**)&sc.grange[1], h.grange[1].data(), h.grange[1].size() * sizeof(Int2)},
            {(void**)&sc.pl_e[0], h.pl_e[0].data(), h.pl_e[0].size() * sizeof(UInt2)},
            {(void**)&sc.pl_e[1], h.pl_e[1].data(), h.pl_e[1].size() * sizeof(UInt2)},
        };
        for (const auto& l : lists) {
            if (hipMalloc(l.dev, l.bytes) != hipSuccess) { tli_free_map(m); return TLI_ERR_ALLOC; }
            if (hipMemcpy(*l.dev, l.host, l.bytes, hipMemcpyHostToDevice) != hipSuccess) { tli_free_map(m); return TLI_ERR_HIP; }
        }
    }
    *out_map = m;
    if (out_num_shared) *out_num_shared = S;
    return TLI_OK;
}

void tli_free_map(tli_map* m) {
    if (!m) return;
    if (m->d2t) (void)hipFree(m->d2t);
    if (m->t2d) (void)hipFree(m->t2d);
    if (m->lmask[0]) (void)hipFree(m->lmask[0]);
    if (m->lmask[1]) (void)hipFree(m->lmask[1]);
    if (m->sh_x) (void)hipFree(m->sh_x);
    if (m->d2r) (void)hipFree(m->d2r);
    if (m->t2r) (void)hipFree(m->t2r);
    for (int dt = 0; dt < 2; ++dt) {
        tli_map::Scan& sc = m->scan[dt];
        void* const owned[] = {sc.cb, sc.part_n, sc.pl_g, sc.stab[0], sc.stab[1], sc.grange[0], sc.grange[1],
                               sc.pl_e[0], sc.pl_e[1]};
        for (void* q : owned)
            if (q) (void)hipFree(q);
    }
    delete m;
}

int tli_map_info(const tli_map* m, int32_t* Vd, int32_t* Vt, int32_t* S) {
    if (!m) return TLI_ERR_INVALID_ARG;
    if (Vd) *Vd = m->Vd;
    if (Vt) *Vt = m->Vt;
    if (S) *S = m->S;
    return TLI_OK;
}

size_t tli_workspace_bytes(int32_t B, int32_t K, int32_t Vt, int32_t Vd, tli_dtype dtype) {
    if (B < 1 || K < 1 || K > kMaxK || !vocab_ok(Vt) || !vocab_ok(Vd) || (dtype != TLI_F32 && dtype != TLI_BF16)) return 0;
    if ((int64_t)B * K > 0x7fffffff / 64) return 0;
    return layout(B, K, Vt, Vd, dtype).total;
}

int tli_draft_sample(const tli_map* map, const void* logits_d, tli_dtype dtype, int64_t row_stride_elems, int32_t R,
                     float temp_d, const float* u_draft, int32_t* tok_d, int32_t* tok_t, double* q_tok, double* lse_q,
                     int32_t* row_status, int64_t io_stride, void* workspace, size_t workspace_bytes,
                     void* hip_stream) {
    if (!map || !tok_t || !lse_q) return TLI_ERR_INVALID_ARG;
    return sample_rows_impl(logits_d, dtype, row_stride_elems, R, map->Vd, temp_d, map->lmask, map->d2t, u_draft, tok_d,
                            tok_t, q_tok, lse_q, row_status, io_stride, workspace, workspace_bytes,
                            static_cast<hipStream_t>(hip_stream));
}

int tli_draft_sample_warped(const tli_map* map, const void* logits_d, tli_dtype dtype, int64_t row_stride_elems,
                            int32_t R, float temp_d, const float* thr, const float* u_draft, int32_t* tok_d,
                            int32_t* tok_t, double* q_tok, double* lse_q, int32_t* row_status, int64_t io_stride,
                            void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!map || !tok_t || !lse_q || !thr) return TLI_ERR_INVALID_ARG;
    return sample_rows_impl(logits_d, dtype, row_stride_elems, R, map->Vd, temp_d, map->lmask, map->d2t, u_draft, tok_d,
                            tok_t, q_tok, lse_q, row_status, io_stride, workspace, workspace_bytes,
                            static_cast<hipStream_t>(hip_stream), nullptr, thr);
}

int tli_draft_sample_compact(const tli_map* map, const void* logits_c, tli_dtype dtype, int64_t row_stride_elems,
                             int32_t R, float temp_d, const float* u_draft, int32_t* tok_d, int32_t* tok_t, double* q_tok,
                             double* lse_q, int32_t* row_status, int64_t io_stride, void* workspace,
                             size_t workspace_bytes, void* hip_stream) {
    if (!map || !tok_t || !lse_q) return TLI_ERR_INVALID_ARG;
    return sample_rows_impl(logits_c, dtype, row_stride_elems, R, map->S, temp_d, nullptr, map->d2t, u_draft, tok_d, tok_t,
                            q_tok, lse_q, row_status, io_stride, workspace, workspace_bytes,
                            static_cast<hipStream_t>(hip_stream), map->sh_x);
}

int tli_union_draft_sample(const tli_map* map, const void* logits_d, tli_dtype dtype, int64_t row_stride_elems,
                           int32_t R, float temp_d, const float* u_draft, int32_t* tok_d, int32_t* tok_t,
                           double* q_tok, double* lse_q, int32_t* row_status, int64_t io_stride, void* workspace,
                           size_t workspace_bytes, void* hip_stream) {
    if (!map || !tok_t || !lse_q) return TLI_ERR_INVALID_ARG;
    return sample_rows_impl(logits_d, dtype, row_stride_elems, R, map->Vd, temp_d, nullptr, map->d2t, u_draft, tok_d,
                            tok_t, q_tok, lse_q, row_status, io_stride, workspace, workspace_bytes,
                            static_cast<hipStream_t>(hip_stream));
}

size_t tli_acceptance_rates_workspace_bytes(const tli_map* map, int32_t B, int32_t K, tli_dtype dtype) {
    if (!map || B < 1 || K < 1 || (int64_t)B * K > 0x7fffffff / 64 || (dtype != TLI_F32 && dtype != TLI_BF16)) return 0;
    return diag_layout(map, B, K, dtype).total;
}

int tli_acceptance_rates(const tli_map* map, const void* logits_t, const void* logits_d, tli_dtype dtype, int32_t B,
                         int32_t K, float temp_t, float temp_d, double* alpha_tli, double* alpha_union,
                         int32_t* pos_status, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!map || !logits_t || !logits_d || !alpha_tli || !alpha_union || !pos_status || !workspace)
        return TLI_ERR_INVALID_ARG;
    if (B < 1 || K < 1 || (int64_t)B * K > 0x7fffffff / 64) return TLI_ERR_INVALID_ARG;
    if (!(temp_t > 0.f) || !(temp_d > 0.f) || !std::isfinite(temp_t) || !std::isfinite(temp_d)) return TLI_ERR_INVALID_ARG;
    if (dtype != TLI_F32 && dtype != TLI_BF16) return TLI_ERR_INVALID_ARG;
    const int epv = dtype == TLI_BF16 ? 8 : 4;
    if (map->Vt % epv != 0 || map->Vd % epv != 0 || !aligned16(logits_t) || !aligned16(logits_d) || !aligned16(workspace))
        return TLI_ERR_INVALID_ARG;
    const DiagLayout w = diag_layout(map, B, K, dtype);
    if (workspace_bytes < w.total) return TLI_ERR_ALLOC;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (dtype == TLI_BF16)
        launch_diag<TLI_BF16>(map, logits_t, logits_d, B, K, temp_t, temp_d, alpha_tli, alpha_union, pos_status,
                              static_cast<char*>(workspace), w, st);
    else
        launch_diag<TLI_F32>(map, logits_t, logits_d, B, K, temp_t, temp_d, alpha_tli, alpha_union, pos_status,
                             static_cast<char*>(workspace), w, st);
    return hipGetLastError() == hipSuccess ? TLI_OK : TLI_ERR_HIP;
}

size_t tli_warp_workspace_bytes(int32_t R, int32_t V, tli_dtype dtype) {
    if (R < 1 || R > 0x7fffffff / 64 || !vocab_ok(V) || (dtype != TLI_F32 && dtype != TLI_BF16)) return 0;
    return align256((size_t)R * sizeof(WarpRow));
}

int tli_warp_rows(const tli_map* map, const void* logits, tli_dtype dtype, int64_t row_stride_elems, int32_t R, int32_t V,
                  float temp, int32_t top_k, float top_p, void* logits_out, int64_t out_stride_elems, float* thr,
                  int32_t* kept, int32_t* row_status, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!logits || !row_status || !workspace) return TLI_ERR_INVALID_ARG;
    if (!logits_out && (kept || !thr)) return TLI_ERR_INVALID_ARG;  // thresholds only: they are the result
    if (R < 1 || R > 0x7fffffff / 64 || !vocab_ok(V) || !(temp > 0.f) || !std::isfinite(temp)) return TLI_ERR_INVALID_ARG;
    if (!(top_p > 0.f) || (map && V != map->Vd)) return TLI_ERR_INVALID_ARG;
    if (dtype != TLI_F32 && dtype != TLI_BF16) return TLI_ERR_INVALID_ARG;
    const int epv = dtype == TLI_BF16 ? 8 : 4;
    if (row_stride_elems < V || row_stride_elems % epv != 0 || !aligned16(logits) || !aligned16(workspace))
        return TLI_ERR_INVALID_ARG;
    if (logits_out && (out_stride_elems < V || out_stride_elems % epv != 0 || !aligned16(logits_out)))
        return TLI_ERR_INVALID_ARG;
    if (workspace_bytes < tli_warp_workspace_bytes(R, V, dtype)) return TLI_ERR_ALLOC;
    const int chunk = dtype == TLI_BF16 ? chunk_elems<TLI_BF16>() : chunk_elems<TLI_F32>();
    const int nC = (V + chunk - 1) / chunk;
    WarpRow* st = reinterpret_cast<WarpRow*>(workspace);
    const double c_true = kLog2e / (double)temp;
    const float cs = (float)c_true;
    const double ratio = c_true / (double)cs;
    const int use_p = top_p < 1.f ? 1 : 0;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const dim3 rows_grid(R);
    // One sweep of the rows per launch: the normaliser with top-k's first digit; top-k's middle digit (three-digit
    // keys); top-k's last digit with the start of top-p; what is left of top-p (rows that have nothing left to
    // decide at a level leave at once); the rewrite, if asked for.
#define TLI_WARP_RUN(DT, MASKED, BITS)                                                                                   \
    do {                                                                                                                  \
        hipLaunchKernelGGL((k_warp_first<DT, MASKED>), rows_grid, dim3(kWG), 0, s, logits, row_stride_elems, V, nC, cs,   \
                           ratio, BITS, top_k, use_p, st);                                                                \
        if (top_k > 0) {                                                                                                  \
            for (int level = 1; level < WarpKey<DT>::LEVELS - 1; ++level)                                                 \
                hipLaunchKernelGGL((k_warp_level<DT, MASKED, 0>), rows_grid, dim3(kWG), 0, s, logits, row_stride_elems,   \
                                   V, nC, level, top_p, c_true, BITS, st);                                                \
            hipLaunchKernelGGL((k_warp_klast<DT, MASKED>), rows_grid, dim3(kWG), 0, s, logits, row_stride_elems, V, nC,   \
                               top_p, c_true, BITS, st);                                                                  \
        }                                                                                                                 \
        if (use_p)                                                                                                        \
            for (int level = 0; level < WarpKey<DT>::LEVELS; ++level)                                                     \
                hipLaunchKernelGGL((k_warp_level<DT, MASKED, 1>), rows_grid, dim3(kWG), 0, s, logits, row_stride_elems,   \
                                   V, nC, level, top_p, c_true, BITS, st);                                                \
        if (logits_out)                                                                                                   \
            hipLaunchKernelGGL((k_warp_apply<DT, MASKED>), rows_grid, dim3(kWG), 0, s, logits, row_stride_elems, V, nC,   \
                               BITS, st, logits_out, out_stride_elems, thr, kept, row_status);                            \
        else                                                                                                              \
            hipLaunchKernelGGL(k_warp_finish<DT>, dim3((R + kWG - 1) / kWG), dim3(kWG), 0, s, st, R, thr, row_status);    \
    } while (0)
    if (map) {
        if (dtype == TLI_BF16) TLI_WARP_RUN(TLI_BF16, true, map->lmask[TLI_BF16]);
        else TLI_WARP_RUN(TLI_F32, true, map->lmask[TLI_F32]);
    } else {
        if (dtype == TLI_BF16) TLI_WARP_RUN(TLI_BF16, false, (const uint64_t*)nullptr);
        else TLI_WARP_RUN(TLI_F32, false, (const uint64_t*)nullptr);
    }
#undef TLI_WARP_RUN
    return hipGetLastError() == hipSuccess ? TLI_OK : TLI_ERR_HIP;
}

size_t tli_sample_rows_workspace_bytes(int32_t R, int32_t V, tli_dtype dtype) {
    if (R < 1 || R > 0x7fffffff / 64 || !vocab_ok(V) || (dtype != TLI_F32 && dtype != TLI_BF16)) return 0;
    return rows_workspace(R, V, dtype);
}

int tli_sample_rows(const void* logits, tli_dtype dtype, int64_t row_stride_elems, int32_t R, int32_t V, float temp,
                    const float* u, int32_t* tok, double* p_tok, double* lse, int32_t* row_status, int64_t io_stride,
                    void* workspace, size_t workspace_bytes, void* hip_stream) {
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (temp == 0.f)
        return argmax_rows_impl(logits, dtype, row_stride_elems, R, V, nullptr, nullptr, tok, nullptr, p_tok, lse,
                                row_status, io_stride, workspace, workspace_bytes, st);
    return sample_rows_impl(logits, dtype, row_stride_elems, R, V, temp, nullptr, nullptr, u, tok, nullptr, p_tok, lse,
                            row_status, io_stride, workspace, workspace_bytes, st);
}

int tli_sample_rows_warped(const void* logits, tli_dtype dtype, int64_t row_stride_elems, int32_t R, int32_t V, float temp,
                           const float* thr, const float* u, int32_t* tok, double* p_tok, double* lse,
                           int32_t* row_status, int64_t io_stride, void* workspace, size_t workspace_bytes,
                           void* hip_stream) {
    if (!thr) return TLI_ERR_INVALID_ARG;
    return sample_rows_impl(logits, dtype, row_stride_elems, R, V, temp, nullptr, nullptr, u, tok, nullptr, p_tok, lse,
                            row_status, io_stride, workspace, workspace_bytes, static_cast<hipStream_t>(hip_stream),
                            nullptr, thr);
}

int tli_greedy_draft(const tli_map* map, const void* logits_d, tli_dtype dtype, int64_t row_stride_elems, int32_t R,
                     int32_t* tok_d, int32_t* tok_t, int32_t* row_status, int64_t io_stride, void* workspace,
                     size_t workspace_bytes, void* hip_stream) {
    if (!map || !tok_t) return TLI_ERR_INVALID_ARG;
    return argmax_rows_impl(logits_d, dtype, row_stride_elems, R, map->Vd, map->lmask, map->d2t, tok_d, tok_t, nullptr,
                            nullptr, row_status, io_stride, workspace, workspace_bytes,
                            static_cast<hipStream_t>(hip_stream));
}

int tli_exact_match_verify(const void* logits_t, tli_dtype dtype, int32_t B, int32_t m, int32_t Vt, float temp_t,
                           const int32_t* draft_t, const float* u, int32_t* n_accepted, int32_t* out_tok,
                           int32_t* tgt_tok, int32_t* seq_status, void* workspace, size_t workspace_bytes,
                           void* hip_stream) {
    if (!logits_t || !draft_t || !n_accepted || !out_tok || !tgt_tok || !seq_status || !workspace)
        return TLI_ERR_INVALID_ARG;
    if (B < 1 || m < 1 || m >= kMaxK || (int64_t)B * (m + 1) > 0x7fffffff / 64 || !vocab_ok(Vt)) return TLI_ERR_INVALID_ARG;
    if (!(temp_t >= 0.f) || !std::isfinite(temp_t) || (temp_t > 0.f && !u)) return TLI_ERR_INVALID_ARG;
    if (dtype != TLI_F32 && dtype != TLI_BF16) return TLI_ERR_INVALID_ARG;
    const int epv = dtype == TLI_BF16 ? 8 : 4;
    if (Vt % epv != 0 || !aligned16(workspace)) return TLI_ERR_INVALID_ARG;  // dense rows must start on 16 bytes
    const int R = B * (m + 1);
    const size_t st_bytes = align256((size_t)R * sizeof(int32_t));
    if (workspace_bytes < st_bytes + rows_workspace(R, Vt, dtype)) return TLI_ERR_ALLOC;
    int32_t* row_status = reinterpret_cast<int32_t*>(workspace);
    void* ws_rows = static_cast<char*>(workspace) + st_bytes;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const int rc = tli_sample_rows(logits_t, dtype, Vt, R, Vt, temp_t, u, tgt_tok, nullptr, nullptr, row_status, 1, ws_rows,
                                   workspace_bytes - st_bytes, st);
    if (rc != TLI_OK) return rc;
    hipLaunchKernelGGL(k_match, dim3(B), dim3(kWave), 0, st, tgt_tok, row_status, draft_t, m, n_accepted, out_tok,
                       seq_status);
    return hipGetLastError() == hipSuccess ? TLI_OK : TLI_ERR_HIP;
}

size_t tli_exact_match_workspace_bytes(int32_t B, int32_t m, int32_t Vt, tli_dtype dtype) {
    if (B < 1 || m < 1 || m >= kMaxK || (int64_t)B * (m + 1) > 0x7fffffff / 64 || !vocab_ok(Vt) ||
        (dtype != TLI_F32 && dtype != TLI_BF16))
        return 0;
    const int R = B * (m + 1);
    return align256((size_t)R * sizeof(int32_t)) + rows_workspace(R, Vt, dtype);
}

static int verify_impl(int union_mode, int64_t compact_stride, const tli_map* map, const void* logits_t,
                       const void* logits_d, tli_dtype dtype, int32_t B, int32_t K, float temp_t, float temp_d, const int32_t* tok_d, const double* lse_q,
                       const float* u_acc, const float* u_fin, int32_t* n_accepted, int32_t* out_tok, uint8_t* accept,
                       double* p_tok, double* q_tok, double* lse_p, int32_t* seq_status, void* workspace,
                       size_t workspace_bytes, void* hip_stream) {
    if (!map || !logits_t || !logits_d || !tok_d || !u_acc || !u_fin || !n_accepted || !out_tok ||
        !seq_status || !workspace)
        return TLI_ERR_INVALID_ARG;
    if (B < 1 || K < 1 || K > kMaxK || (int64_t)B * K > 0x7fffffff / 64) return TLI_ERR_INVALID_ARG;
    if (!(temp_t > 0.f) || !(temp_d > 0.f) || !std::isfinite(temp_t) || !std::isfinite(temp_d))
        return TLI_ERR_INVALID_ARG;
    if (dtype != TLI_F32 && dtype != TLI_BF16) return TLI_ERR_INVALID_ARG;
    const int epv = dtype == TLI_BF16 ? 8 : 4;
    const int Vt = map->Vt, Vd = map->Vd;
    const bool compact = compact_stride != 0;
    // dense rows must each start on a 16-byte boundary; compact drafter rows: S valid entries, compact_stride apart
    if (Vt % epv != 0 || !aligned16(logits_t) || !aligned16(logits_d) || !aligned16(workspace)) return TLI_ERR_INVALID_ARG;
    if (compact ? (compact_stride < map->S || compact_stride % epv != 0) : (Vd % epv != 0)) return TLI_ERR_INVALID_ARG;
    const Workspace w = layout(B, K, Vt, Vd, dtype);
    if (workspace_bytes < w.total) return TLI_ERR_ALLOC;
    char* ws = static_cast<char*>(workspace);
    Part* part = reinterpret_cast<Part*>(ws + w.part);
    float* tab_ref = reinterpret_cast<float*>(ws + w.tab_ref);
    float* tab_s = reinterpret_cast<float*>(ws + w.tab_s);
    const int chunk = dtype == TLI_BF16 ? chunk_elems<TLI_BF16>() : chunk_elems<TLI_F32>();
    const int rows = B * K;
    const Plan pl = make_plan(Vt, rows, chunk);
    const Plan pf = make_plan(Vt, B, chunk);
    const double c_t = kLog2e / (double)temp_t, c_d = kLog2e / (double)temp_d;
    const float cs_t = (float)c_t;
    const double ratio_t = c_t / (double)cs_t;
    const double inv_t = 1.0 / (double)temp_t, inv_d = 1.0 / (double)temp_d;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    VerifyArgs a;
    a.map = map; a.logits_t = logits_t; a.logits_d = logits_d; a.B = B; a.K = K; a.pl = pl; a.pf = pf;
    a.c_t = c_t; a.c_d = c_d; a.cs_t = cs_t; a.ratio_t = ratio_t; a.inv_t = inv_t; a.inv_d = inv_d;
    a.tok_d = tok_d; a.lse_q = lse_q; a.u_acc = u_acc; a.u_fin = u_fin; a.n_accepted = n_accepted;
    a.out_tok = out_tok; a.accept = accept; a.p_tok = p_tok; a.q_tok = q_tok; a.lse_p = lse_p;
    a.seq_status = seq_status; a.part = part;
    a.part_d = reinterpret_cast<Part*>(ws + w.part_d); a.ws_lse_q = reinterpret_cast<double*>(ws + w.ws_lse_q);
    a.compact = compact ? 1 : 0;
    a.d_valid = compact ? map->S : Vd;
    a.dv.base = logits_d;
    a.dv.row_stride = compact ? compact_stride : (int64_t)Vd;
    a.dv.d2x = compact ? map->d2r : nullptr;
    a.dv.t2x = compact ? map->t2r : map->t2d;
    a.pd = make_plan(a.d_valid, rows, chunk); a.cs_d = (float)c_d; a.ratio_d = c_d / (double)a.cs_d; a.tab_ref = tab_ref; a.tab_s = tab_s;
    a.rmass = reinterpret_cast<double*>(ws + w.rmass); a.fbad = reinterpret_cast<int32_t*>(ws + w.fbad); a.ctab = reinterpret_cast<float2*>(ws + w.ctab);
    a.frow = reinterpret_cast<FinalRow*>(ws + w.frow);
    a.union_mode = union_mode;
    if (dtype == TLI_BF16) launch_verify<TLI_BF16>(a, st);
    else launch_verify<TLI_F32>(a, st);
    return hipGetLastError() == hipSuccess ? TLI_OK : TLI_ERR_HIP;
}

int tli_verify(const tli_map* map, const void* logits_t, const void* logits_d, tli_dtype dtype, int32_t B, int32_t K,
               float temp_t, float temp_d, const int32_t* tok_d, const double* lse_q, const float* u_acc,
               const float* u_fin, int32_t* n_accepted, int32_t* out_tok, uint8_t* accept, double* p_tok,
               double* q_tok, double* lse_p, int32_t* seq_status, void* workspace, size_t workspace_bytes,
               void* hip_stream) {
    return verify_impl(0, 0, map, logits_t, logits_d, dtype, B, K, temp_t, temp_d, tok_d, lse_q, u_acc, u_fin, n_accepted,
                       out_tok, accept, p_tok, q_tok, lse_p, seq_status, workspace, workspace_bytes, hip_stream);
}

size_t tli_verify_static_max_bytes(void) { return kStaticScratchBytes; }

int tli_verify_static(const tli_map* map, const void* logits_t, const void* logits_d, tli_dtype dtype, int32_t B, int32_t K,
                      float temp_t, float temp_d, const int32_t* tok_d, const double* lse_q, const float* u_acc,
                      const float* u_fin, int32_t* n_accepted, int32_t* out_tok, uint8_t* accept, double* p_tok,
                      double* q_tok, double* lse_p, int32_t* seq_status, void* hip_stream) {
    if (!map) return TLI_ERR_INVALID_ARG;
    const size_t need = tli_workspace_bytes(B, K, map->Vt, map->Vd, dtype);
    if (need == 0) return TLI_ERR_INVALID_ARG;
    if (need > kStaticScratchBytes) return TLI_ERR_TOO_LARGE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return TLI_ERR_HIP;
    if (dev != map->device) return TLI_ERR_INVALID_ARG;  // the map's tables and the scratch must be on the current device
    void* ws = nullptr;
    const int rc = static_scratch(dev, &ws);
    if (rc != TLI_OK) return rc;
    // Nothing in the scratch has to start at zero: every kernel of the call writes what a later one reads (the
    // per-sequence flag is reset by the accept kernel), so the previous call's contents are simply overwritten.
    return verify_impl(0, 0, map, logits_t, logits_d, dtype, B, K, temp_t, temp_d, tok_d, lse_q, u_acc, u_fin, n_accepted,
                       out_tok, accept, p_tok, q_tok, lse_p, seq_status, ws, kStaticScratchBytes, hip_stream);
}

int tli_verify_compact(const tli_map* map, const void* logits_t, const void* logits_c, int64_t c_row_stride_elems,
                       tli_dtype dtype, int32_t B, int32_t K, float temp_t, float temp_d, const int32_t* tok_d,
                       const double* lse_q, const float* u_acc, const float* u_fin, int32_t* n_accepted, int32_t* out_tok,
                       uint8_t* accept, double* p_tok, double* q_tok, double* lse_p, int32_t* seq_status, void* workspace,
                       size_t workspace_bytes, void* hip_stream) {
    if (c_row_stride_elems < 1) return TLI_ERR_INVALID_ARG;
    return verify_impl(0, c_row_stride_elems, map, logits_t, logits_c, dtype, B, K, temp_t, temp_d, tok_d, lse_q, u_acc,
                       u_fin, n_accepted, out_tok, accept, p_tok, q_tok, lse_p, seq_status, workspace, workspace_bytes,
                       hip_stream);
}

int tli_union_verify(const tli_map* map, const void* logits_t, const void* logits_d, tli_dtype dtype, int32_t B,
                     int32_t K, float temp_t, float temp_d, const int32_t* tok_d, const double* lse_q,
                     const float* u_acc, const float* u_fin, int32_t* n_accepted, int32_t* out_tok, uint8_t* accept,
                     double* p_tok, double* q_tok, double* lse_p, int32_t* seq_status, void* workspace,
                     size_t workspace_bytes, void* hip_stream) {
    return verify_impl(1, 0, map, logits_t, logits_d, dtype, B, K, temp_t, temp_d, tok_d, lse_q, u_acc, u_fin, n_accepted,
                       out_tok, accept, p_tok, q_tok, lse_p, seq_status, workspace, workspace_bytes, hip_stream);
}

}  // extern "C"
