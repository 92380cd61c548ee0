// tli_next_kernels.h -- Neighbours of the hot path: expected acceptance rates, temperature zero (argmax), the exact-matching tail,
// top-k / top-p logit warpers, and the copy kernel that calibrates hardware byte counters.  Included by
// tli_kernels.hip inside its unnamed namespace, after tli_verify_kernels.h.
#pragma once

// ---- expected acceptance rates of every position ------------------------------------------------
// Table of expected acceptance rates: alpha_union = sum_{T∩D} min{p, q}, alpha_tli = sum_{T∩D} min{p, q'} with
// q' = q / sum_{T∩D} q; the theorem on the intersection algorithm states alpha_union <= alpha_tli.
// A workgroup's partial normaliser from the (ref, s) pairs its waves parked in LDS (+ a wave's running total of the
// chunks that did not fit there).  Called by all threads, after a barrier; ends with one.
__device__ __forceinline__ void finish_partial(const float2* stash, int n_here, const Running& over, double kd,
                                               float* sref, double* ssum, Part* out) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float r_mine = over.ref;
    for (int i = threadIdx.x; i < n_here; i += kWG) r_mine = fmaxf(r_mine, stash[i].x);
    r_mine = wave_max(r_mine);
    if (lane == 0) sref[wave] = r_mine;
    __syncthreads();
    float R = sref[0];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) R = fmaxf(R, sref[w]);
    double s_mine = lane == 0 ? over.s * exp2_diff(over.ref, R, kd) : 0.0;  // a wave's overflow total counts once
    for (int i = threadIdx.x; i < n_here; i += kWG) {
        const float2 e = stash[i];
        s_mine += (double)e.y * exp2_diff(e.x, R, kd);
    }
    s_mine = wave_sum_f64(s_mine);
    if (lane == 0) ssum[wave] = s_mine;
    __syncthreads();
    if (threadIdx.x == 0) {
        double S = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) S += ssum[w];
        Part p; p.ref = R; p.pad = 0.f; p.s = S;
        *out = p;
    }
    __syncthreads();
}

// kernel: both drafter normalisers of every position in one pass over the drafter rows -- over the shared ids
// (q' of the intersection algorithm, part_sh) and over all of D (q of the union algorithm, part_all).
// grid (rows * nsplit), as k_lse.
template <int DT>
__global__ __launch_bounds__(kWG) void k_lse_both(const void* __restrict__ logits, int K, int64_t seq_stride,
                                                   int64_t row_stride, int V, int nC, int cps, int nsplit, float cs,
                                                   double ratio, const uint64_t* __restrict__ bits,
                                                   Part* __restrict__ part_sh, Part* __restrict__ part_all) {
    const int row = blockIdx.x / nsplit, split = blockIdx.x - row * nsplit;
    const int b = row / K, k = row - b * K;
    const u4v* rowv = reinterpret_cast<const u4v*>(static_cast<const char*>(logits) +
                                                    (b * seq_stride + k * row_stride) * Traits<DT>::ESZ);
    const int lane = threadIdx.x & 63;
    const double kd = (ratio - 1.0) * kLn2;
    const float dl = (float)(ratio - 1.0);
    __shared__ float2 stash_all[kLdsChunks], stash_sh[kLdsChunks];
    __shared__ float sref[kWaves];
    __shared__ double ssum[kWaves];
    Running over_all, over_sh;
    const int c0 = split * cps, c1 = min(nC, (split + 1) * cps);
    stream_chunks<DT, kWaves>(rowv, V, c0, c1, [&](const ChunkRegs& r, int c, auto whole) {
        float ref, s_all, ref_sh, s_sh;
        bool ok;
        reduce_chunk_both<DT, decltype(whole)::value>(r, c, lane, V, cs, dl, bits, ref, s_all, s_sh, ok);
        ref_sh = ref;
        if (!ok) reduce_chunk<DT, true, decltype(whole)::value>(r, c, lane, V, cs, dl, bits, ref_sh, s_sh);
        const int i = c - c0;
        if (i < kLdsChunks) {
            if (lane == 0) {
                stash_all[i] = make_float2(ref, s_all);
                stash_sh[i] = make_float2(ref_sh, s_sh);
            }
        } else {
            over_all.add(ref, s_all, kd);
            over_sh.add(ref_sh, s_sh, kd);
        }
    });
    __syncthreads();
    const int n_here = min(c1 - c0, kLdsChunks);
    finish_partial(stash_all, n_here, over_all, kd, sref, ssum, part_all + (int64_t)row * nsplit + split);
    finish_partial(stash_sh, n_here, over_sh, kd, sref, ssum, part_sh + (int64_t)row * nsplit + split);
}

// kernel: one record per position (b, k) from the three normalisers (target row, drafter row over the
// shared ids, drafter row over all of D).  grid (ceil(rows / 256)).
__global__ __launch_bounds__(kWG) void k_diag_rows(const Part* __restrict__ part_t, int nsplit_t,
                                                    const Part* __restrict__ part_q1, const Part* __restrict__ part_q2,
                                                    int nsplit_d, int rows, int K, double ratio_t, double ratio_d,
                                                    double c_t, double c_d, FinalRow* __restrict__ frow,
                                                    int32_t* __restrict__ fbad, int32_t* __restrict__ status) {
    const int r = blockIdx.x * kWG + threadIdx.x;
    if (r >= rows) return;
    const int b = r / K, k = r - b * K;
    const double lp = combine_parts(part_t + (int64_t)r * nsplit_t, nsplit_t, ratio_t);
    const double lq1 = combine_parts(part_q1 + (int64_t)r * nsplit_d, nsplit_d, ratio_d);
    const double lq2 = combine_parts(part_q2 + (int64_t)r * nsplit_d, nsplit_d, ratio_d);
    const bool nonfinite = lp != lp || lq2 != lq2 || lq1 != lq1;
    FinalRow f;
    f.skip = nonfinite ? 1 : 0;
    f.bonus = 0;
    f.n = k;
    f.t_row = b * (K + 1) + k;
    f.d_row = r;
    f.dq = f.dq_lo = 0.f;
    f.l2p = 0.0;
    f.rp.use_q = 0;
    f.rp.ct_hi = f.rp.ct_lo = f.rp.lp_hi = f.rp.lp_lo = 0.f;
    f.rp.cd_hi = f.rp.cd_lo = f.rp.lq_hi = f.rp.lq_lo = 0.f;
    if (!nonfinite && lp > -INFINITY && lq1 > -INFINITY) {
        f.rp.use_q = 1;
        f.l2p = lp * kLog2e;
        split_scale(c_t, f.rp.ct_hi, f.rp.ct_lo);
        split_hi_lo(f.l2p, f.rp.lp_hi, f.rp.lp_lo);
        split_scale(c_d, f.rp.cd_hi, f.rp.cd_lo);
        split_hi_lo(lq1 * kLog2e, f.rp.lq_hi, f.rp.lq_lo);
        split_hi_lo((lq2 - lq1) * kLog2e, f.dq, f.dq_lo);
    }
    frow[r] = f;
    fbad[r] = 0;
    status[r] = nonfinite ? TLI_FLAG_NONFINITE : (lq1 == -INFINITY ? TLI_FLAG_ZERO_MASS : 0);
}

// kernel: alpha of every position = sum over parts and chunks of the scan's partial sums.  grid (rows), one wave.
// pass 0 (after the fp32 scan) also marks in redo the positions with a rate below 2^-24: their terms lie where the
// fp32 scan's exponent arguments and range no longer give 1e-5; pass 1 (after the fp64-argument scan of those
// positions) rewrites only them.
__global__ __launch_bounds__(kWave) void k_diag_finish(const FinalRow* __restrict__ frow, const double* __restrict__ mn,
                                                        const double* __restrict__ mn2, int rows, int nC,
                                                        double* __restrict__ alpha_tli, double* __restrict__ alpha_union,
                                                        int32_t* __restrict__ redo, int pass) {
    const int r = blockIdx.x, lane = threadIdx.x;
    if (pass == 1 && !redo[r]) return;
    const FinalRow f = frow[r];
    double a1 = 0.0, a2 = 0.0;
    if (f.skip) {
        a1 = a2 = NAN;
    } else if (f.rp.use_q) {
        const double* m1 = mn + (int64_t)r * nC;
        const double* m2 = mn2 + (int64_t)r * nC;
        for (int c = lane; c < nC; c += kWave) { a1 += m1[c]; a2 += m2[c]; }
        a1 = wave_sum_f64(a1);
        a2 = wave_sum_f64(a2);
    }
    if (lane == 0) {
        alpha_tli[r] = a1;
        alpha_union[r] = a2;
        if (pass == 0) redo[r] = (!f.skip && f.rp.use_q && (a1 < 0x1p-24 || a2 < 0x1p-24)) ? 1 : 0;
    }
}

// ---- temperature zero: argmax of rows ----------------------------------------------------------
// At temperature zero every draw of the path becomes an argmax (the paper runs its exact-matching method
// that way): the largest logit, the lowest id among equal ones.  Same streaming scan as the softmax
// kernels.  Per chunk a lane only takes the maximum of its 32 elements and remembers the chunk it came
// from; the id is found at the end by re-reading that one chunk (4 vectors per lane).  MASKED: only the
// shared ids compete (greedy TLI draft).  NaN or +inf among the competing logits flags the row.
struct ArgPart {  // best of (a split of) a row
    float v;
    int32_t idx;   // -1: nothing competes / everything -inf
    int32_t bad;   // a competing logit is NaN or +inf
    int32_t pad;
};

template <int DT, bool MASKED>
__global__ __launch_bounds__(kWG) void k_argmax(const void* __restrict__ logits, int64_t row_stride, int V, int nC,
                                                 int cps, int nsplit, const uint64_t* __restrict__ bits,
                                                 ArgPart* __restrict__ part) {
    constexpr int EPV = Traits<DT>::EPV;
    constexpr int N = EPV * kLoads;
    const int row = blockIdx.x / nsplit, split = blockIdx.x - row * nsplit;
    const char* rowp = static_cast<const char*>(logits) + (int64_t)row * row_stride * Traits<DT>::ESZ;
    const u4v* rowv = reinterpret_cast<const u4v*>(rowp);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    float best = -INFINITY;
    int bc = -1;
    bool bad = false;
    stream_chunks<DT, kWaves>(rowv, V, split * cps, min(nC, (split + 1) * cps), [&](const ChunkRegs& r, int c, auto whole) {
        float x[N];
        chunk_values<DT, MASKED, decltype(whole)::value>(r, c, lane, V, bits, x);
        float m = x[0];
        bool nan = x[0] != x[0];
#pragma unroll
        for (int i = 1; i < N; ++i) {
            m = fmaxf(m, x[i]);
            nan |= x[i] != x[i];
        }
        bad |= nan;
        if (m > best) { best = m; bc = c; }  // strict: an equal maximum in a later chunk has a higher id
    });
    bad |= best == INFINITY;
    // wave: the largest value, then the lowest id among the lanes that hold it.  Only those lanes (one, or a
    // few on ties) look their id up: the first element equal to the maximum in the chunk the lane took it
    // from.  That chunk differs from lane to lane, so the shared-id mask is taken per lane here (mask_bits),
    // not as a wave-wide word.
    const float M = wave_max(best);
    int cand = 0x7fffffff;
    if (bc >= 0 && best == M) {
        const int64_t nvec = (V + EPV - 1) / EPV;
#pragma unroll
        for (int j = kLoads - 1; j >= 0; --j) {
            const int64_t vi = ((int64_t)bc * kLoads + j) * kWave + lane;
            if (vi >= nvec) continue;
            float x[EPV];
            unpack<DT>(reinterpret_cast<const uint4*>(rowp)[vi], x);
            const uint32_t mb = MASKED ? mask_bits<DT>(bits, vi) : 0xffu;
#pragma unroll
            for (int i = EPV - 1; i >= 0; --i)
                if (vi * EPV + i < V && ((mb >> i) & 1u) && x[i] == best) cand = (int)(vi * EPV + i);
        }
    }
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) cand = min(cand, __shfl_xor(cand, d, kWave));
    const bool wbad = __ballot(bad) != 0ull;
    __shared__ float sv[kWaves];
    __shared__ int si[kWaves], sb[kWaves];
    if (lane == 0) { sv[wave] = M; si[wave] = cand; sb[wave] = wbad ? 1 : 0; }
    __syncthreads();
    if (threadIdx.x == 0) {
        ArgPart a;
        a.v = -INFINITY; a.idx = 0x7fffffff; a.bad = 0; a.pad = 0;
        for (int w = 0; w < kWaves; ++w) {
            a.bad |= sb[w];
            if (sv[w] > a.v || (sv[w] == a.v && si[w] < a.idx)) { a.v = sv[w]; a.idx = si[w]; }
        }
        if (a.idx == 0x7fffffff) a.idx = -1;
        part[(int64_t)row * nsplit + split] = a;
    }
}

// kernel: argmax of every row from the partials of its splits.  grid (ceil(rows / 256)).
// tok[r] = id (or -1), tok_t[r] = d2t[id] if both given, p_tok = 1, status = NONFINITE / ZERO_MASS / 0;
// entry of row r at index r * io_stride.
__global__ __launch_bounds__(kWG) void k_argmax_finish(const ArgPart* __restrict__ part, int rows, int nsplit,
                                                        const int32_t* __restrict__ d2t, int32_t* __restrict__ tok,
                                                        int32_t* __restrict__ tok_t, double* __restrict__ p_tok,
                                                        double* __restrict__ lse, int32_t* __restrict__ status,
                                                        int64_t io_stride) {
    const int row = blockIdx.x * kWG + threadIdx.x;
    if (row >= rows) return;
    const ArgPart* pr = part + (int64_t)row * nsplit;
    ArgPart a = pr[0];
    for (int sidx = 1; sidx < nsplit; ++sidx) {
        const ArgPart b = pr[sidx];
        a.bad |= b.bad;
        if (b.idx >= 0 && (a.idx < 0 || b.v > a.v || (b.v == a.v && b.idx < a.idx))) { a.v = b.v; a.idx = b.idx; }
    }
    const int64_t at = (int64_t)row * io_stride;
    const int st = a.bad ? TLI_FLAG_NONFINITE : (a.idx < 0 || a.v == -INFINITY ? TLI_FLAG_ZERO_MASS : 0);
    const int id = st ? -1 : a.idx;
    tok[at] = id;
    if (tok_t) tok_t[at] = (id >= 0 && d2t) ? d2t[id] : id;
    if (p_tok) p_tok[at] = st ? 0.0 : 1.0;
    if (lse) lse[at] = NAN;
    status[at] = st;
}

// ---- kernel: first mismatch between the target's own tokens and the re-tokenised draft -----------
// Exact-matching verification (string-level exact match, its last two steps): j* = first j with
// t'_j != draft_j, output draft_1..draft_{j*-1}, t'_{j*}.  grid (B), 64 threads; lane j owns position j.
__global__ __launch_bounds__(kWave) void k_match(const int32_t* __restrict__ tgt_tok, const int32_t* __restrict__ row_status,
                                                  const int32_t* __restrict__ draft_t, int m,
                                                  int32_t* __restrict__ n_accepted, int32_t* __restrict__ out_tok,
                                                  int32_t* __restrict__ seq_status) {
    const int b = blockIdx.x, j = threadIdx.x;
    int st = 0, tt = -1, dr = -1;
    if (j <= m) {
        st = row_status[(int64_t)b * (m + 1) + j];
        tt = tgt_tok[(int64_t)b * (m + 1) + j];
    }
    if (j < m) dr = draft_t[(int64_t)b * m + j];
    int any = st;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) any |= __shfl_xor(any, d, kWave);
    const bool differs = (j < m) ? (dr < 0 || dr != tt) : (j == m);
    const unsigned long long mism = __ballot(differs);
    const int n = any ? 0 : (int)__builtin_ctzll(mism);  // bit m is always set
    if (j <= m) out_tok[(int64_t)b * (m + 1) + j] = any ? -1 : (j < n ? dr : (j == n ? tt : -1));
    if (j == 0) { n_accepted[b] = n; seq_status[b] = any; }
}

// ---- logit warpers ahead of the softmax: top-k and top-p by value thresholds -----------------------
// The paper samples at plain temperature (or temperature zero); these are the standard serving knobs around
// the same softmax.  Both are defined by a threshold on the logit VALUE, so equal logits are kept or dropped
// together and nothing depends on a sort order:
//   top-k: keep logits >= the k-th largest competing logit;
//   top-p: on what survived top-k (renormalised), keep x iff the mass of strictly larger logits is < top_p.
// The threshold is found by a most-significant-digit-first radix descent over an order-preserving integer key
// of the logit (16 bits for bf16: two 8-bit digits; 32 bits for fp32: digits of 11, 11 and 10 bits).  Each
// level is one pass over the rows: a workgroup per row histograms the digit of the elements whose higher
// digits match the prefix found so far -- element counts (top-k) and probability mass (top-p, in 2^-48 fixed
// point so that sums do not depend on the order of arrival) -- and then picks the digit in which the
// threshold lies.  Logits crowd into a handful of leading digits (sign and exponent), so the lanes of a wave
// would queue on the same few LDS words: the histogram is kept in several interleaved copies, one per lane
// group, and folded after the scan.  A last pass writes the rows with every dropped logit set to -inf (or only
// the thresholds are returned).
// Passes that can share a sweep of the rows do: the first digit of top-k is counted while the row's normaliser
// is formed (k_warp_first), and the sweep for top-k's last digit also gathers what top-p needs to start among
// the survivors -- their mass per first digit -- so that top-p's first digit (and, for two-digit keys, its second
// whenever it falls in top-k's own bin) is decided there too (k_warp_klast).  Top-k 50 + top-p 0.9 on bf16 rows
// is then two sweeps and the rewrite instead of six.
constexpr int kWarpBinsMax = 2048;
constexpr double kMassScale = 281474976710656.0;  // 2^48
template <int DT> struct WarpKey;
template <> struct WarpKey<TLI_BF16> {
    static constexpr int LEVELS = 2;
    static constexpr int COPIES = 16;  // private copies of the histogram (lane & 15 picks one), interleaved per bin
    static constexpr int BINS = 256;
    __host__ __device__ static constexpr int bits(int) { return 8; }
    __host__ __device__ static constexpr int shift(int level) { return level == 0 ? 8 : 0; }
};
template <> struct WarpKey<TLI_F32> {
    static constexpr int LEVELS = 3;
    static constexpr int COPIES = 2;
    static constexpr int BINS = 2048;
    __host__ __device__ static constexpr int bits(int level) { return level == 2 ? 10 : 11; }
    __host__ __device__ static constexpr int shift(int level) { return level == 0 ? 21 : (level == 1 ? 10 : 0); }
};

// order-preserving key of a logit given as fp32 bits (bf16 logits arrive widened: only the top 16 bits are used);
// -0 is folded onto +0 so that equal values share a key
template <int DT> __device__ __forceinline__ uint32_t warp_key(float x) {
    uint32_t u = as_u(x);
    if (u == 0x80000000u) u = 0u;
    const uint32_t k = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return DT == TLI_BF16 ? (k >> 16) : k;
}
template <int DT> __device__ __forceinline__ float warp_unkey(uint32_t k) {
    if (DT == TLI_BF16) k <<= 16;
    const uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return as_f(DT == TLI_BF16 ? (u & 0xffff0000u) : u);
}

struct WarpRow {
    double l2;            // log-normaliser of the competing logits, log2 units
    uint64_t zk;          // mass of the logits that survive top-k (2^-48 fixed point)
    uint64_t p_above;     // mass strictly above the top-p prefix found so far
    uint64_t target;      // top_p * zk
    uint32_t kprefix;     // key digits of the top-k threshold found so far (right-aligned)
    uint32_t pprefix;     // same for the top-p threshold
    uint32_t k_rem;       // the threshold is the k_rem-th largest key below the prefix
    int32_t k_on, p_on;   // the warper is active for this row (top-k turns itself off when k >= competing ids)
    int32_t p_level;      // the next digit top-p has to decide (LEVELS: it is through)
    int32_t status;
};

// kernel: the row's normaliser, the start of its state, and -- with top-k on -- the first digit of top-k's
// threshold, from one sweep of the row.  grid (R), 256 threads.
template <int DT, bool MASKED>
__global__ __launch_bounds__(kWG) void k_warp_first(const void* __restrict__ logits, int64_t row_stride, int V, int nC,
                                                     float cs, double ratio, const uint64_t* __restrict__ bits,
                                                     int top_k, int use_p, WarpRow* __restrict__ st) {
    constexpr int EPV = Traits<DT>::EPV;
    constexpr int N = EPV * kLoads;
    constexpr int COPIES = WarpKey<DT>::COPIES;
    constexpr int nbits = WarpKey<DT>::bits(0), shift = WarpKey<DT>::shift(0), nbins = 1 << nbits;
    const int row = blockIdx.x;
    __shared__ uint32_t cnt_c[WarpKey<DT>::BINS * COPIES];
    const bool count = top_k > 0;
    if (count)
        for (int i = threadIdx.x; i < nbins * COPIES; i += kWG) cnt_c[i] = 0u;
    __syncthreads();
    const int copy = threadIdx.x & (COPIES - 1);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const double kd = (ratio - 1.0) * kLn2;
    const float dl = (float)(ratio - 1.0);
    const u4v* rowv = reinterpret_cast<const u4v*>(static_cast<const char*>(logits) + (int64_t)row * row_stride * Traits<DT>::ESZ);
    Running run;
    stream_chunks<DT, kWaves>(rowv, V, 0, nC, [&](const ChunkRegs& r, int c, auto whole) {
        float x[N];
        chunk_values<DT, MASKED, decltype(whole)::value>(r, c, lane, V, bits, x);
        float ref, sum;
        reduce_values<N>(x, cs, dl, ref, sum);
        run.add(ref, sum, kd);
        if (count) {
#pragma unroll
            for (int i = 0; i < N; ++i)
                if (x[i] > -INFINITY)
                    atomicAdd(&cnt_c[((warp_key<DT>(x[i]) >> shift) & (uint32_t)(nbins - 1)) * COPIES + copy], 1u);
        }
    });
    __shared__ Part sp[kWaves];
    __shared__ uint32_t cnt[WarpKey<DT>::BINS];
    if (lane == 0) { sp[wave].ref = run.ref; sp[wave].pad = 0.f; sp[wave].s = run.s; }
    __syncthreads();
    if (count)
        for (int i = threadIdx.x; i < nbins; i += kWG) {  // fold the copies
            uint32_t c = 0;
#pragma unroll
            for (int k = 0; k < COPIES; ++k) c += cnt_c[i * COPIES + k];
            cnt[i] = c;
        }
    __syncthreads();
    if (threadIdx.x != 0) return;
    const double lse = combine_parts(sp, kWaves, ratio);
    WarpRow w;
    w.l2 = lse * kLog2e;
    w.zk = 0; w.p_above = 0; w.target = 0; w.kprefix = 0; w.pprefix = 0;
    w.k_rem = top_k > 0 ? (uint32_t)top_k : 0u;
    w.status = lse != lse ? TLI_FLAG_NONFINITE : (lse == -INFINITY ? TLI_FLAG_ZERO_MASS : 0);
    w.k_on = (top_k > 0 && !w.status) ? 1 : 0;
    w.p_on = (use_p && !w.status) ? 1 : 0;
    w.p_level = 0;
    if (w.k_on) {
        // no more competing ids than k: top-k drops nothing and turns itself off; else the digit d with
        // #above(d) < k <= #above(d) + cnt[d], from the top
        uint32_t total = 0;
        for (int d = 0; d < nbins; ++d) total += cnt[d];
        if (total <= w.k_rem) {
            w.k_on = 0;
        } else {
            uint32_t ac = 0;
            int d = nbins - 1;
            while (ac + cnt[d] < w.k_rem) ac += cnt[d--];  // ends: the total exceeds k
            w.kprefix = (uint32_t)d;
            w.k_rem -= ac;
        }
    }
    st[row] = w;
}

// kernel: one level of the radix descent.  MODE 0: top-k (counts, and the mass that survives); MODE 1: top-p.
// grid (R), 256 threads.
template <int DT, bool MASKED, int MODE>
__global__ __launch_bounds__(kWG) void k_warp_level(const void* __restrict__ logits, int64_t row_stride, int V, int nC,
                                                     int level, float top_p, double c_true,
                                                     const uint64_t* __restrict__ bits, WarpRow* __restrict__ st) {
    constexpr int EPV = Traits<DT>::EPV;
    constexpr int N = EPV * kLoads;
    const int row = blockIdx.x;
    WarpRow w = st[row];
    if (MODE == 0 ? !w.k_on : (!w.p_on || w.p_level != level)) return;
    const int nbits = WarpKey<DT>::bits(level), shift = WarpKey<DT>::shift(level), nbins = 1 << nbits;
    const uint32_t prefix = MODE == 0 ? w.kprefix : w.pprefix;
    constexpr int COPIES = WarpKey<DT>::COPIES;
    constexpr int kSlots = WarpKey<DT>::BINS * COPIES;
    __shared__ uint32_t cnt_c[kSlots];
    __shared__ unsigned long long mass_c[kSlots];
    __shared__ uint32_t cnt[WarpKey<DT>::BINS];
    __shared__ unsigned long long mass[WarpKey<DT>::BINS];
    for (int i = threadIdx.x; i < nbins * COPIES; i += kWG) { cnt_c[i] = 0u; mass_c[i] = 0ull; }
    const int copy = threadIdx.x & (COPIES - 1);
    __shared__ unsigned long long zk_all;  // mass of the logits that survived top-k
    if (threadIdx.x == 0) zk_all = 0ull;
    unsigned long long zk_mine = 0ull;
    __syncthreads();
    float ch, cl, lh, ll;
    split_scale(c_true, ch, cl);
    split_hi_lo(w.l2, lh, ll);
    const u4v* rowv = reinterpret_cast<const u4v*>(static_cast<const char*>(logits) + (int64_t)row * row_stride * Traits<DT>::ESZ);
    const int lane = threadIdx.x & 63;
    stream_chunks<DT, kWaves>(rowv, V, 0, nC, [&](const ChunkRegs& r, int c, auto whole) {
        float x[N];
        chunk_values<DT, MASKED, decltype(whole)::value>(r, c, lane, V, bits, x);
#pragma unroll
        for (int i = 0; i < N; ++i) {
            if (!(x[i] > -INFINITY)) continue;  // dropped, masked out or past the end: does not compete
            const uint32_t key = warp_key<DT>(x[i]);
            if (level > 0 && (key >> (shift + nbits)) != prefix) continue;
            // top-p is decided among the survivors of top-k: with top-k on, nothing below its threshold can matter
            if (MODE == 1 && w.k_on && key < w.kprefix) continue;
            const uint32_t d = (key >> shift) & (uint32_t)(nbins - 1);
            if (MODE == 0) {  // top-k only counts; the mass that survives it is summed by the first top-p pass
                atomicAdd(&cnt_c[d * COPIES + copy], 1u);
            } else {
                const float pr = exp2_split(x[i], ch, cl, lh, ll);
                const unsigned long long fx = (unsigned long long)((double)pr * kMassScale);
                atomicAdd(&mass_c[d * COPIES + copy], fx);
                if (level == 0 && w.k_on && key >= w.kprefix) zk_mine += fx;
            }
        }
    });
    if (MODE == 1 && level == 0 && w.k_on) {  // integer sums: the order of arrival does not matter
#pragma unroll
        for (int dd = 1; dd < kWave; dd <<= 1) zk_mine += __shfl_xor(zk_mine, dd, kWave);
        if (lane == 0) atomicAdd(&zk_all, zk_mine);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nbins; i += kWG) {  // fold the copies (integer sums: any order gives the same result)
        uint32_t c = 0;
        unsigned long long m = 0;
#pragma unroll
        for (int k = 0; k < COPIES; ++k) { c += cnt_c[i * COPIES + k]; m += mass_c[i * COPIES + k]; }
        cnt[i] = c; mass[i] = m;
    }
    __syncthreads();
    // suffix sums over the bins (from the top): thread t owns bins [t*per, (t+1)*per)
    const int per = nbins / kWG > 0 ? nbins / kWG : 1;
    const int t = threadIdx.x;
    uint32_t my_c = 0;
    unsigned long long my_m = 0;
    if (t * per < nbins)
        for (int i = 0; i < per; ++i) { my_c += cnt[t * per + i]; my_m += mass[t * per + i]; }
    __shared__ uint32_t tc[kWG];
    __shared__ unsigned long long tm[kWG];
    tc[t] = my_c; tm[t] = my_m;
    __syncthreads();
    // counts and mass in the bins of all higher threads (a short serial loop: 256 entries)
    uint32_t above_c = 0;
    unsigned long long above_m = 0;
    for (int u = t + 1; u < kWG; ++u) { above_c += tc[u]; above_m += tm[u]; }
    __shared__ unsigned long long total_m;
    __shared__ uint32_t total_c;
    __shared__ int best_d;
    if (t == 0) { total_m = above_m + my_m; total_c = above_c + my_c; best_d = 0x7fffffff; }
    __syncthreads();
    const bool owns = t * per < nbins;
    if (MODE == 0) {
        if (level == 0 && total_c <= w.k_rem) {
            // no more competing ids than k: top-k drops nothing, everything survives
            if (t == 0) st[row].k_on = 0;
            return;
        }
        // the digit d with  #above(d) < k_rem <= #above(d) + cnt[d]  (exactly one thread finds it)
        uint32_t ac = above_c;
        for (int i = per - 1; owns && i >= 0; --i) {
            const int d = t * per + i;
            if (ac < w.k_rem && w.k_rem <= ac + cnt[d]) {
                WarpRow& o = st[row];
                o.kprefix = (prefix << nbits) | (uint32_t)d;
                o.k_rem = w.k_rem - ac;
            }
            ac += cnt[d];
        }
    } else {
        unsigned long long target = w.target;
        if (level == 0) {
            const unsigned long long z = w.k_on ? zk_all : total_m;
            target = (unsigned long long)((double)top_p * (double)z);
            if (t == 0) { st[row].target = target; st[row].zk = z; }
        }
        // the lowest digit d with mass whose strictly-above mass is still below the target
        unsigned long long am = w.p_above + above_m;
        int found = -1;
        unsigned long long found_am = 0;
        for (int i = per - 1; owns && i >= 0; --i) {
            const int d = t * per + i;
            if (mass[d] > 0ull && am < target) { found = d; found_am = am; }
            am += mass[d];
        }
        // several threads may hold candidates: the lowest digit wins (the condition is monotone in the digit)
        if (found >= 0) atomicMin(&best_d, found);
        __syncthreads();
        if (found >= 0 && found == best_d) {
            WarpRow& o = st[row];
            o.pprefix = (prefix << nbits) | (uint32_t)found;
            o.p_above = found_am;
        }
        if (t == 0) st[row].p_level = level + 1;
    }
}

// kernel: the last digit of top-k's threshold and, from the same sweep, the start of top-p among the survivors.
// Beside the counts of the last digit under top-k's prefix the sweep gathers the mass per FIRST digit of the elements
// above the prefix whose first digit is larger than the prefix's, and the mass of the rest above the prefix
// (three-digit keys only); those elements are fewer than k, so their histogram needs no copies and the branch that
// forms a mass is rarely taken.  The elements under the prefix need none formed one by one: a last digit fixes the
// whole key, so the mass of a bin is its count times the mass of that one value.  Once the threshold is known these
// give the mass that survives top-k, top-p's target, its first digit, and -- for two-digit keys, when that digit is
// top-k's own -- its second.  grid (R), 256 threads.
template <int DT, bool MASKED>
__global__ __launch_bounds__(kWG) void k_warp_klast(const void* __restrict__ logits, int64_t row_stride, int V, int nC,
                                                     float top_p, double c_true, const uint64_t* __restrict__ bits,
                                                     WarpRow* __restrict__ st) {
    constexpr int EPV = Traits<DT>::EPV;
    constexpr int N = EPV * kLoads;
    constexpr int L = WarpKey<DT>::LEVELS, level = L - 1;
    constexpr int nbits = WarpKey<DT>::bits(level), nbins = 1 << nbits;  // the last digit sits at shift 0
    constexpr int nbits0 = WarpKey<DT>::bits(0), shift0 = WarpKey<DT>::shift(0), nbins0 = 1 << nbits0;
    constexpr int COPIES = WarpKey<DT>::COPIES;
    const int row = blockIdx.x;
    const WarpRow w = st[row];
    if (!w.k_on) return;
    const uint32_t prefix = w.kprefix;                        // the digits above the last
    const uint32_t k0 = prefix >> (shift0 - nbits);           // the first of them
    const bool use_p = w.p_on != 0;
    __shared__ uint32_t cnt_c[nbins * COPIES];
    __shared__ uint32_t cnt[nbins];
    __shared__ unsigned long long mass[nbins];
    __shared__ unsigned long long mass0[nbins0];
    __shared__ unsigned long long mid;
    for (int i = threadIdx.x; i < nbins * COPIES; i += kWG) cnt_c[i] = 0u;
    for (int i = threadIdx.x; i < nbins0; i += kWG) mass0[i] = 0ull;
    if (threadIdx.x == 0) mid = 0ull;
    __syncthreads();
    const int copy = threadIdx.x & (COPIES - 1);
    const int lane = threadIdx.x & 63;
    float ch, cl, lh, ll;
    split_scale(c_true, ch, cl);
    split_hi_lo(w.l2, lh, ll);
    unsigned long long mid_mine = 0ull;
    const u4v* rowv = reinterpret_cast<const u4v*>(static_cast<const char*>(logits) + (int64_t)row * row_stride * Traits<DT>::ESZ);
    stream_chunks<DT, kWaves>(rowv, V, 0, nC, [&](const ChunkRegs& r, int c, auto whole) {
        float x[N];
        chunk_values<DT, MASKED, decltype(whole)::value>(r, c, lane, V, bits, x);
#pragma unroll
        for (int i = 0; i < N; ++i) {
            if (!(x[i] > -INFINITY)) continue;
            const uint32_t key = warp_key<DT>(x[i]);
            const uint32_t hp = key >> nbits;
            if (hp < prefix) continue;  // below the threshold whatever its last digit is
            if (hp == prefix) {
                atomicAdd(&cnt_c[(key & (uint32_t)(nbins - 1)) * COPIES + copy], 1u);
            } else if (use_p) {  // above the threshold: a survivor
                const unsigned long long fx = (unsigned long long)((double)exp2_split(x[i], ch, cl, lh, ll) * kMassScale);
                const uint32_t d0 = key >> shift0;
                if (d0 > k0) atomicAdd(&mass0[d0], fx);
                else mid_mine += fx;
            }
        }
    });
    if (L > 2 && use_p) {
#pragma unroll
        for (int dd = 1; dd < kWave; dd <<= 1) mid_mine += __shfl_xor(mid_mine, dd, kWave);
        if (lane == 0 && mid_mine) atomicAdd(&mid, mid_mine);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nbins; i += kWG) {
        uint32_t c = 0;
#pragma unroll
        for (int k = 0; k < COPIES; ++k) c += cnt_c[i * COPIES + k];
        cnt[i] = c;
        unsigned long long m = 0ull;
        if (use_p && c) {  // every element of the bin has the key (prefix, i): c equal masses
            const float xv = warp_unkey<DT>((prefix << nbits) | (uint32_t)i);
            m = (unsigned long long)c * (unsigned long long)((double)exp2_split(xv, ch, cl, lh, ll) * kMassScale);
        }
        mass[i] = m;
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    // top-k: the last digit.  At least k_rem elements lie under the prefix (that is how the prefix was chosen).
    uint32_t ac = 0;
    int dk = nbins - 1;
    while (dk > 0 && ac + cnt[dk] < w.k_rem) ac += cnt[dk--];
    WarpRow o = w;
    o.kprefix = (prefix << nbits) | (uint32_t)dk;
    o.k_rem = w.k_rem - ac;
    if (use_p) {
        unsigned long long surv = 0ull, above0 = 0ull;
        for (int d = nbins - 1; d >= dk; --d) surv += mass[d];
        for (int d0 = nbins0 - 1; d0 > (int)k0; --d0) above0 += mass0[d0];
        const unsigned long long here = mid + surv;  // the survivors whose first digit is top-k's
        o.zk = above0 + here;
        o.target = (unsigned long long)((double)top_p * (double)o.zk);
        // top-p's first digit: the lowest one with mass whose strictly-above mass is still below the target
        unsigned long long am = 0ull, found_am = 0ull;
        int found = -1;
        for (int d0 = nbins0 - 1; d0 > (int)k0; --d0) {
            if (mass0[d0] > 0ull && am < o.target) { found = d0; found_am = am; }
            am += mass0[d0];
        }
        if (here > 0ull && am < o.target) { found = (int)k0; found_am = am; }
        if (found < 0) {  // no survivor carries mass at this resolution: top-p has nothing to decide
            o.pprefix = 0u; o.p_above = 0ull; o.p_level = L;
        } else if (found > (int)k0 || L > 2) {
            o.pprefix = (uint32_t)found; o.p_above = found_am; o.p_level = 1;
        } else {  // two-digit keys, top-k's own first digit: the survivors there are the digits >= dk counted above
            unsigned long long am1 = found_am, f1_am = found_am;
            int f1 = dk;
            for (int d = nbins - 1; d >= dk; --d) {
                if (mass[d] > 0ull && am1 < o.target) { f1 = d; f1_am = am1; }
                am1 += mass[d];
            }
            o.pprefix = (k0 << nbits) | (uint32_t)f1; o.p_above = f1_am; o.p_level = L;
        }
    }
    st[row] = o;
}

// kernel: thresholds and flags without the rewrite.  The threshold is the lowest value that is kept: top-p's if it
// lies above top-k's, else top-k's, else -inf (no warper active for the row).  grid (ceil(R / 256)).
template <int DT>
__global__ __launch_bounds__(kWG) void k_warp_finish(const WarpRow* __restrict__ st, int R, float* __restrict__ thr,
                                                      int32_t* __restrict__ status) {
    const int r = blockIdx.x * kWG + threadIdx.x;
    if (r >= R) return;
    const WarpRow w = st[r];
    uint32_t tkey = 0;
    bool any = false;
    if (w.k_on) { tkey = w.kprefix; any = true; }
    if (w.p_on && (!any || w.pprefix > tkey)) { tkey = w.pprefix; any = true; }
    if (thr) thr[r] = w.status ? NAN : (any ? warp_unkey<DT>(tkey) : -INFINITY);
    status[r] = w.status;
}

// kernel: write the warped rows (dropped logits = -inf), thresholds and survivor counts.  grid (R), 256 threads.
template <int DT, bool MASKED>
__global__ __launch_bounds__(kWG) void k_warp_apply(const void* __restrict__ logits, int64_t row_stride, int V, int nC,
                                                     const uint64_t* __restrict__ bits, const WarpRow* __restrict__ st,
                                                     void* __restrict__ out, int64_t out_stride, float* __restrict__ thr,
                                                     int32_t* __restrict__ kept, int32_t* __restrict__ status) {
    constexpr int EPV = Traits<DT>::EPV;
    const int row = blockIdx.x;
    const WarpRow w = st[row];
    uint32_t tkey = 0;  // keep everything that competes
    bool any = false;
    if (w.k_on) { tkey = w.kprefix; any = true; }
    if (w.p_on && (!any || w.pprefix > tkey)) { tkey = w.pprefix; any = true; }
    const u4v* rowv = reinterpret_cast<const u4v*>(static_cast<const char*>(logits) + (int64_t)row * row_stride * Traits<DT>::ESZ);
    uint4* dst = reinterpret_cast<uint4*>(static_cast<char*>(out) + (int64_t)row * out_stride * Traits<DT>::ESZ);
    const int nvec = (V + EPV - 1) / EPV;
    const unsigned int npat = (DT == TLI_BF16) ? 0xff80u : 0xff800000u;
    const int lane = threadIdx.x & 63;
    int n = 0, n_k = 0;  // survivors of both warpers; survivors of top-k alone (all competing ids if it is off)
    stream_chunks<DT, kWaves>(rowv, V, 0, nC, [&](const ChunkRegs& r, int c, auto) {
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            const int vi = (c * kLoads + j) * kWave + lane;
            if (vi >= nvec) continue;
            const uint4 in = to_uint4(r.v[j]);
            float x[EPV];
            unpack<DT>(in, x);
            const uint32_t mb = MASKED ? mask_bits<DT>(bits, vi) : 0xffu;
            uint32_t o[EPV];
#pragma unroll
            for (int i = 0; i < EPV; ++i) {
                const bool competes = vi * EPV + i < V && ((mb >> i) & 1u) && !w.status && x[i] > -INFINITY;
                const uint32_t key = warp_key<DT>(x[i]);
                const bool live = competes && (!any || key >= tkey);
                n += live ? 1 : 0;
                n_k += (competes && (!w.k_on || key >= w.kprefix)) ? 1 : 0;
                o[i] = live ? (DT == TLI_BF16 ? as_u(x[i]) >> 16 : as_u(x[i])) : npat;
            }
            uint32_t nw[4];
            if constexpr (DT == TLI_BF16) {
                nw[0] = o[0] | (o[1] << 16); nw[1] = o[2] | (o[3] << 16); nw[2] = o[4] | (o[5] << 16); nw[3] = o[6] | (o[7] << 16);
            } else {
                nw[0] = o[0]; nw[1] = o[1]; nw[2] = o[2]; nw[3] = o[3];
            }
            // the last vector of a row whose length is not a multiple of the vector keeps the caller's padding
            if ((vi + 1) * EPV > V) {
                const uint32_t kw[4] = {in.x, in.y, in.z, in.w};
#pragma unroll
                for (int i = 0; i < EPV; ++i)
                    if (vi * EPV + i >= V) {
                        if constexpr (DT == TLI_BF16) {
                            const uint32_t sh = (i & 1) * 16;
                            nw[i >> 1] = (nw[i >> 1] & ~(0xffffu << sh)) | (kw[i >> 1] & (0xffffu << sh));
                        } else {
                            nw[i] = kw[i];
                        }
                    }
            }
            dst[vi] = make_uint4(nw[0], nw[1], nw[2], nw[3]);
        }
    });
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) { n += __shfl_xor(n, d, kWave); n_k += __shfl_xor(n_k, d, kWave); }
    __shared__ int sn[kWaves], snk[kWaves];
    if ((threadIdx.x & 63) == 0) { sn[threadIdx.x >> 6] = n; snk[threadIdx.x >> 6] = n_k; }
    __syncthreads();
    if (threadIdx.x == 0) {
        int tot = 0, tot_k = 0;
        for (int i = 0; i < kWaves; ++i) { tot += sn[i]; tot_k += snk[i]; }
        if (kept) kept[row] = tot;
        // the threshold reported is the value that decided: top-p's only if it dropped something that top-k had
        // kept, else top-k's (the k-th largest logit), else -inf
        const float th = tot < tot_k ? warp_unkey<DT>(tkey) : (w.k_on ? warp_unkey<DT>(w.kprefix) : -INFINITY);
        if (thr) thr[row] = w.status ? NAN : th;
        status[row] = w.status;
    }
}

// ---- plain copy, used only to calibrate hardware byte counters against a known size -----------
__global__ __launch_bounds__(kWG) void k_calib_copy(const u4v* __restrict__ src, u4v* __restrict__ dst, size_t nvec) {
    const size_t stride = (size_t)gridDim.x * kWG;
    for (size_t i = (size_t)blockIdx.x * kWG + threadIdx.x; i < nvec; i += stride) dst[i] = src[i];
}

// ---- plain read, the yardstick the streaming kernels are held against ---------------------------------
// Reads `slabs` contiguous slabs of `slab_vec` 16-byte vectors, a workgroup per slab, in the normaliser kernel's
// own access pattern (a wave owns chunks of 64 lanes x 4 loads, the next chunk's loads in flight) and does
// nothing with the data but fold it into one word per workgroup, so that the loads cannot be dropped.
template <bool NT>
__global__ __launch_bounds__(kWG) void k_calib_read(const u4v* __restrict__ src, size_t slab_vec, uint32_t* __restrict__ out) {
    const u4v* base = src + (size_t)blockIdx.x * slab_vec;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const size_t nchunks = slab_vec / (kWave * kLoads);
    u4v acc = {0u, 0u, 0u, 0u};
    auto load = [&](size_t c, u4v (&v)[kLoads]) {
        const u4v* q = base + c * (kWave * kLoads) + lane;
#pragma unroll
        for (int j = 0; j < kLoads; ++j) v[j] = NT ? __builtin_nontemporal_load(q + j * kWave) : q[j * kWave];
    };
    auto fold = [&](const u4v (&v)[kLoads]) {
#pragma unroll
        for (int j = 0; j < kLoads; ++j) acc ^= v[j];
    };
    size_t c = wave;
    if (c < nchunks) {
        u4v a[kLoads], b[kLoads];
        load(c, a);
        for (; c + kWaves < nchunks; c += kWaves) {
            load(c + kWaves, b);
            fold(a);
#pragma unroll
            for (int j = 0; j < kLoads; ++j) a[j] = b[j];
        }
        fold(a);
    }
    const uint32_t w = acc.x ^ acc.y ^ acc.z ^ acc.w;
    if (w == 0x9e3779b9u) out[blockIdx.x] = w;  // practically never: the store only keeps the loads alive
}
