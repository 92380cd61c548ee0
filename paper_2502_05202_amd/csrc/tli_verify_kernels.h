// tli_verify_kernels.h -- Verification: accept tests and first-reject scan, the residual distribution of the rejected position (chunk
// masses, then the draw), the bonus row.  Included by tli_kernels.hip inside its unnamed namespace, after
// tli_softmax_kernels.h.
#pragma once

// ---- how the verification kernels address the drafter logits ------------------------------------
// Full layout: rows of Vd logits in drafter-id order.  Compact layout (a drafter head pruned to the shared
// tokens): rows of S logits in rank order (rank = position among the shared ids, ascending drafter id).
struct DrafterView {
    const void* base;
    int64_t row_stride;    // elements between consecutive rows
    const int32_t* d2x;    // drafter id -> index in a row; nullptr = identity (full layout)
    const int32_t* t2x;    // target id -> index in a row, -1 for target-only ids (t2d full, t2r compact)
};

// ---- what the final kernels need to know about a sequence, written once by the accept kernel ----
struct ResidualParams {
    float ct_hi, ct_lo, lp_hi, lp_lo;  // target: p = 2^(x*ct - Lp), Lp = lse_p * log2 e
    float cd_hi, cd_lo, lq_hi, lq_lo;  // drafter: q' = 2^(y*cd - Lq)
    int use_q;                         // 0: the rejected draft was unusable, q' = 0 everywhere
};
struct FinalRow {
    int skip;       // sequence is flagged NONFINITE
    int bonus;      // nothing rejected: sample from p of row K
    int n;          // accepted count = index of the row the extra token comes from
    int t_row;      // that row in the target tensor (dense row index), and its partner in the drafter tensor
    int d_row;
    float dq;       // diagnostics only: log2 q'(x) - log2 q(x) = (lse_q over D - lse_q over T∩D) * log2 e >= 0
    ResidualParams rp;
    float dq_lo;    // what dq's rounding to fp32 left out (the wide form of the diagnostic scan adds it back)
    double l2p;     // lse_p of row n, in log2 units
};

__device__ __forceinline__ void split_hi_lo(double v, float& hi, float& lo) {
    hi = (float)v;
    lo = (float)(v - (double)hi);
}

// scale c > 0 as hi + lo with hi < c, so that lo > 0
__device__ __forceinline__ void split_scale(double c, float& hi, float& lo) {
    hi = (float)c;
    if ((double)hi >= c) hi = as_f(as_u(hi) - 1u);
    lo = (float)(c - (double)hi);
}

// ---- accept tests and first-reject scan of one sequence ------------------------------------------
// Standard SD appendix, verification loop and the count of accepted drafts, from the normaliser partials of the
// sequence's K target rows.  One wave, lane k owns position k.  Returns the sequence's record for the extra-token
// step, the same in every lane; if `write`, also stores the sequence's outputs and that record.
struct AcceptIn {
    const Part* part;  // [B*K][nsplit] partial normalisers of the target rows
    int nsplit;
    double ratio_t, inv_temp_t, inv_temp_d, c_t, c_d;
    const int32_t *d2t, *tok_d;
    const double* lse_q;
    const float* u_acc;
    int union_mode;
};
struct AcceptOut {
    int32_t *n_accepted, *out_tok;
    uint8_t* accept;
    double *p_tok, *q_tok, *lse_p;
    int32_t* seq_status;
    FinalRow* frow;
};

template <int DT>
__device__ __forceinline__ FinalRow accept_sequence(int b, const void* __restrict__ logits_t, const DrafterView& dv, int K,
                                                    int Vt, int Vd, const AcceptIn& in, const AcceptOut& out, bool write) {
    const int k = threadIdx.x & 63;
    bool acc = true, nonfinite = false, bad = false;
    int tt = -1;
    double my_lse = 0.0, my_lq = 0.0;
    if (k < K) {
        const int64_t row = (int64_t)b * K + k;
        // The draft's two logits are at the end of a chain of three dependent loads (draft, its target id, the
        // logits): it is started before the partials are combined, not after.
        const int d = in.tok_d[row];
        my_lq = in.lse_q[row];
        const float u = in.u_acc[row];
        const bool d_ok = d >= 0 && d < Vd;
        const int td = d_ok ? in.d2t[d] : -1;
        // TLI: a draft must be a shared drafter id.  Union algorithm: any drafter id is a legal draft; one
        // outside T has target probability 0 and is rejected by the test itself; every drafter logit takes
        // part there, so a NaN normaliser (NaN/+inf somewhere in the row) flags the sequence.
        bad = !d_ok || (!in.union_mode && td < 0);
        float xt = 0.f, xd = 0.f;
        if (!bad) {
            const char* lt = static_cast<const char*>(logits_t) + ((int64_t)b * (K + 1) + k) * Vt * Traits<DT>::ESZ;
            const char* ld = static_cast<const char*>(dv.base) + row * dv.row_stride * Traits<DT>::ESZ;
            if (td >= 0) xt = load_elem<DT>(lt, td);
            xd = load_elem<DT>(ld, dv.d2x ? dv.d2x[d] : d);
        }
        const double lse = combine_parts(in.part + row * in.nsplit, in.nsplit, in.ratio_t);
        nonfinite = lse != lse;
        my_lse = lse;
        double pd = 0.0, qd = 0.0;
        acc = false;
        if (bad) {
        } else if (in.union_mode && my_lq != my_lq) {
            nonfinite = true;
        } else if (!nonfinite) {
            tt = td;
            pd = (tt < 0 || lse == -INFINITY) ? 0.0 : exp((double)xt * in.inv_temp_t - lse);
            qd = (in.union_mode && my_lq == -INFINITY) ? 0.0 : exp((double)xd * in.inv_temp_d - my_lq);
            acc = (double)u * qd < pd;
        }
        if (write) {
            if (out.lse_p) out.lse_p[(int64_t)b * (K + 1) + k] = lse;
            if (out.accept) out.accept[row] = acc ? 1 : 0;
            if (out.p_tok) out.p_tok[row] = pd;
            if (out.q_tok) out.q_tok[row] = qd;
        }
    }
    const unsigned long long rej = __ballot(k < K && !acc);
    const bool any_nonfinite = __ballot(nonfinite) != 0ull;
    const bool any_bad = __ballot(bad) != 0ull;
    int n = rej ? (int)__builtin_ctzll(rej) : K;
    if (any_nonfinite) n = 0;
    if (write) {
        if (k < K) out.out_tok[(int64_t)b * (K + 1) + k] = (k < n) ? tt : -1;
        if (k == 0) {
            out.out_tok[(int64_t)b * (K + 1) + K] = -1;
            out.n_accepted[b] = n;
            out.seq_status[b] = (any_nonfinite ? TLI_FLAG_NONFINITE : 0) | (any_bad ? TLI_FLAG_BAD_DRAFT : 0);
            if (out.lse_p) out.lse_p[(int64_t)b * (K + 1) + K] = NAN;
        }
    }
    // the record: what the lane that owns the row the extra token comes from knows, handed to every lane
    const bool residual = !any_nonfinite && n < K;
    const int owner = residual ? n : 0;
    const double o_lse = __shfl(my_lse, owner, kWave), o_lq = __shfl(my_lq, owner, kWave);
    const bool o_bad = __shfl((int)bad, owner, kWave) != 0;
    FinalRow f;
    f.skip = any_nonfinite ? 1 : 0;
    f.bonus = (!any_nonfinite && n == K) ? 1 : 0;
    f.n = n;
    f.t_row = b * (K + 1) + (f.bonus ? K : n);
    f.d_row = b * K + (f.bonus ? 0 : n);
    f.dq = f.dq_lo = 0.f;
    f.l2p = 0.0;
    f.rp.use_q = 0;
    f.rp.ct_hi = f.rp.ct_lo = f.rp.lp_hi = f.rp.lp_lo = 0.f;
    f.rp.cd_hi = f.rp.cd_lo = f.rp.lq_hi = f.rp.lq_lo = 0.f;
    if (residual) {
        f.l2p = o_lse * kLog2e;
        split_scale(in.c_t, f.rp.ct_hi, f.rp.ct_lo);
        split_hi_lo(f.l2p, f.rp.lp_hi, f.rp.lp_lo);
        // an unusable draft, or a drafter row without mass, has q' = 0 everywhere
        if (!o_bad && (o_lq > -INFINITY || o_lq != o_lq)) {
            f.rp.use_q = 1;
            split_scale(in.c_d, f.rp.cd_hi, f.rp.cd_lo);
            split_hi_lo(o_lq * kLog2e, f.rp.lq_hi, f.rp.lq_lo);
        }
    }
    if (write && k == 0) out.frow[b] = f;
    return f;
}

// ---- extra token: weights of one vector of the residual row -----------------------------------
// Standard SD appendix, last step: r(t) ∝ p(t) - min(p(t), q'(t)) = max(0, p(t) - q'(t)); q'(t) is
// the adjusted drafter's probability of the drafter id that maps to t (0 for target-only ids).
// p and q' are evaluated as 2^(x*c - L) with c and L split into fp32 hi + lo parts, so both carry
// about one ulp of error: the difference of two nearly equal probabilities must not inherit the
// rounding of a large exponent.
// 2^(x*(c_hi+c_lo) - (l_hi+l_lo)) with one rounding of each partial product.  c_lo is strictly positive
// (see split_scale), so a -inf logit gives -inf + -inf = -inf (probability 0), never inf - inf.
__device__ __forceinline__ float exp2_split(float x, float c_hi, float c_lo, float l_hi, float l_lo) {
    return exp2_hw(fmaf(x, c_hi, -l_hi) + fmaf(x, c_lo, -l_lo));
}

// The residual weight of a shared target id in the form that stays accurate when q' is close to p:
//     max(0, p - q') = p * (1 - 2^d),  d = log2 q' - log2 p < 0  (0 for d >= 0),
// with d formed in fp64 from the two logits and the two normalisers.  p - q' taken from two fp32 values, each good
// to 1e-7 of itself, is good to 1e-7 of p -- useless once the two models agree to a percent; here the weight keeps
// 1e-7 of ITSELF (p's own error) whatever the distance.  NaN for a NaN or +inf drafter logit (it must surface).
struct ResidualWide {
    double ct, l2p, cd, l2q;  // log2 p = x * ct - l2p, log2 q' = y * cd - l2q
};
__device__ __forceinline__ ResidualWide widen(const ResidualParams& rp, double l2p) {
    ResidualWide w;
    w.ct = (double)rp.ct_hi + (double)rp.ct_lo;
    w.cd = (double)rp.cd_hi + (double)rp.cd_lo;
    w.l2p = l2p;
    w.l2q = (double)rp.lq_hi + (double)rp.lq_lo;
    return w;
}
__device__ __forceinline__ double residual_weight(float p, float xv, float yv, const ResidualWide& rw) {
    if (!(yv <= 3.0e38f)) return NAN;
    if (!(p > 0.f)) return p != p ? NAN : 0.0;
    const double d = fma((double)yv, rw.cd, -rw.l2q) - fma((double)xv, rw.ct, -rw.l2p);
    if (!(d < 0.0)) return 0.0;
    // 1 - 2^d.  Below d = -1 nothing cancels: the hardware exponential's 6e-8 is 6e-8 of the result (d = -inf, a -inf
    // drafter logit, gives 1: the whole of p).  Above, the series of -expm1(z), z = d ln 2 in (-0.7, 0), in fp32 on the
    // fp64 difference (ten terms: z^11/11! < 1e-9; the last steps round values near 1, so the factor keeps ~1e-7).
    // Both are evaluated and one is chosen: no lane waits for another's branch.
    const float fd = (float)d;
    const float far = 1.f - exp2_hw(fd);
    const float z = fd * 0.693147180559945309f;
    // 1 + z/2! + z^2/3! + ... + z^9/10!, by Horner
    float t = 1.f / 3628800.f;
    t = fmaf(t, z, 1.f / 362880.f);
    t = fmaf(t, z, 1.f / 40320.f);
    t = fmaf(t, z, 1.f / 5040.f);
    t = fmaf(t, z, 1.f / 720.f);
    t = fmaf(t, z, 1.f / 120.f);
    t = fmaf(t, z, 1.f / 24.f);
    t = fmaf(t, z, 1.f / 6.f);
    t = fmaf(t, z, 0.5f);
    const float near = -(z * fmaf(t, z, 1.f));
    return (double)p * (double)(fd < -1.f ? far : near);
}

template <int DT>
__device__ __forceinline__ void residual_vec(const void* rowp, int64_t vi, int V, const ResidualParams& rp, double l2p,
                                             const int32_t* __restrict__ t2d, const void* __restrict__ ld_row,
                                             float* p, double* w) {
    constexpr int EPV = Traits<DT>::EPV;
    const int64_t nvec = (V + EPV - 1) / EPV;
    const int64_t vc = vi < nvec ? vi : nvec - 1;
    const int64_t e0 = vi * EPV;
    float x[EPV];
    unpack<DT>(static_cast<const uint4*>(rowp)[vc], x);
    float y[EPV];
    int32_t d[EPV];
    if (rp.use_q) {
#pragma unroll
        for (int i = 0; i < EPV; i += 4) {
            const int4 t = *reinterpret_cast<const int4*>(t2d + vc * EPV + i);  // t2d is padded to a multiple of 8
            d[i] = t.x; d[i + 1] = t.y; d[i + 2] = t.z; d[i + 3] = t.w;
        }
#pragma unroll
        for (int i = 0; i < EPV; ++i) y[i] = load_elem<DT>(ld_row, d[i] > 0 ? d[i] : 0);
    }
    const ResidualWide rw = widen(rp, l2p);
#pragma unroll
    for (int i = 0; i < EPV; ++i) {
        const bool live = e0 + i < V;
        float pi = exp2_split(x[i], rp.ct_hi, rp.ct_lo, rp.lp_hi, rp.lp_lo);
        pi = live ? pi : 0.f;
        p[i] = pi;
        w[i] = (rp.use_q && live && d[i] >= 0) ? residual_weight(pi, x[i], y[i], rw) : (double)pi;
    }
}

// ---- extra token of one sequence from the chunk tables of its row ------------------------------
// Standard SD appendix, last step: writes out_tok[b, n_accepted[b]]; for bonus rows also lse_p[b, K].
struct FinalOut {
    const float* u_fin;
    int32_t *n_accepted, *out_tok;
    double* lse_p;
    int32_t* seq_status;
};

// what the draw of one sequence's extra token came to (the same in every thread of the workgroup)
struct PickResult {
    int tok;         // the token, -1 if there is none
    int add_flags;   // TLI_FLAG_DEGENERATE if the fallback was taken
    bool nonfinite;  // no distribution to draw from: NaN/+inf in a row that takes part, or a bonus row without mass
    double lse_bonus;  // bonus rows: log-normaliser of row K
};

template <int DT>
__device__ __forceinline__ PickResult final_pick_core(const FinalRow& f, int b, const void* logits_t, const DrafterView& dv,
                                                      int K, int Vt, int Vd, int nC, float cs_t, double ratio_t,
                                                      const int32_t* t2d, const float* tr, const float* ts,
                                                      const float2* ctab, const double* rmass, bool drafter_bad,
                                                      double u) {
    constexpr int EPV = Traits<DT>::EPV;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const char* rowp = static_cast<const char*>(logits_t) + (int64_t)f.t_row * Vt * Traits<DT>::ESZ;
    PickResult res;
    res.tok = -1; res.add_flags = 0; res.nonfinite = false; res.lse_bonus = NAN;
    if (f.bonus) {
        float M;
        double total;
        res.tok = sample_softmax_row<DT, false>(rowp, Vt, nC, cs_t, ratio_t, nullptr, tr, ts, u, &M, &total);
        // no usable mass: NaN/+inf, or a bonus row of only -inf -- no distribution to sample either way
        if (res.tok < 0) res.nonfinite = true;
        else res.lse_bonus = kLn2 * ((double)M * ratio_t + log2(total));
        return res;
    }
    const char* ldp = static_cast<const char*>(dv.base) + (int64_t)f.d_row * dv.row_stride * Traits<DT>::ESZ;
    // chunk masses: the scan left them (sum_chunk p - sum of min(p, q'), or formed without that subtraction, see
    // precise_chunk_masses); a row without a usable draft has q' = 0 and its masses are the chunk sums of p, from
    // the normaliser kernel's table of row n
    const float2* crow = ctab + (int64_t)f.d_row * nC;
    // A chunk with mass in the table can still hold no id whose weight shows in fp32: probabilities below 2^-126 flush
    // to zero, and a chunk sum of p less a sum of min(p, q') that should be 0 is rounding noise of either sign.  A
    // draw that lands in one (u = 0 with such a chunk in front; one time in 10^7 or fewer otherwise) takes the chunk
    // out and searches again, instead of returning no token.
    constexpr int kEmptyMax = 4;
    int skip[kEmptyMax];
#pragma unroll
    for (int i = 0; i < kEmptyMax; ++i) skip[i] = -1;
    int nskip = 0;
    auto skipped = [&](int cc) {
        bool s = false;
#pragma unroll
        for (int i = 0; i < kEmptyMax; ++i) s |= cc == skip[i];
        return s;
    };
    auto p_mass = [&](int cc) {
        const float2 rs = crow[cc];
        return (rs.x == -INFINITY || skipped(cc)) ? 0.0 : (double)rs.y * exp2((double)rs.x * ratio_t - f.l2p);
    };
    auto r_mass = [&](int cc) { return f.rp.use_q ? (skipped(cc) ? 0.0 : rmass[cc]) : p_mass(cc); };
    double theta_local, total;
    bool degenerate = false;
    if (f.rp.use_q && drafter_bad) {  // NaN or +inf among the shared drafter logits of row n
        res.nonfinite = true;
        return res;
    }
    for (;;) {
        const int c = degenerate ? find_chunk(nC, u, p_mass, &theta_local, &total) : find_chunk(nC, u, r_mass, &theta_local, &total);
        if (c < 0) {
            if (total != total || degenerate) {  // NaN somewhere, or p has no mass either
                res.nonfinite = true;
                return res;
            }
            // residual identically zero: fall back to p of the same row
            degenerate = true;
            res.add_flags |= TLI_FLAG_DEGENERATE;
#pragma unroll
            for (int i = 0; i < kEmptyMax; ++i) skip[i] = -1;
            nskip = 0;
            continue;
        }
        // wave j of the workgroup takes load j of the chunk: a quarter of the table look-ups, gathers and
        // exponentials each
        const int64_t vi = ((int64_t)c * kLoads + wave) * kWave + lane;
        double wd[EPV];
        if (wave < kLoads) {
            float p[EPV];
            double w[EPV];
            residual_vec<DT>(rowp, vi, Vt, f.rp, f.l2p, t2d, ldp, p, w);
#pragma unroll
            for (int i = 0; i < EPV; ++i) wd[i] = degenerate ? (double)p[i] : w[i];
        } else {  // a larger workgroup's further waves take no part in the draw
#pragma unroll
            for (int i = 0; i < EPV; ++i) wd[i] = 0.0;
        }
        res.tok = chunk_draw<EPV>(wd, vi * EPV, theta_local);  // (the same in every thread)
        if (res.tok >= 0 || nskip == kEmptyMax) break;
#pragma unroll
        for (int i = 0; i < kEmptyMax; ++i)
            if (i == nskip) skip[i] = c;
        ++nskip;
    }
    return res;
}

template <int DT>
__device__ __forceinline__ void final_pick_row(const FinalRow& f, int b, const void* logits_t, const DrafterView& dv,
                                               int K, int Vt, int Vd, int nC, float cs_t, double ratio_t,
                                               const int32_t* t2d, const float* tr, const float* ts,
                                               const float2* ctab, const double* rmass, bool drafter_bad,
                                               const FinalOut& o) {
    const PickResult r = final_pick_core<DT>(f, b, logits_t, dv, K, Vt, Vd, nC, cs_t, ratio_t, t2d, tr, ts, ctab, rmass,
                                             drafter_bad, (double)o.u_fin[b]);
    if (threadIdx.x == 0) {
        if (r.nonfinite) {
            o.n_accepted[b] = 0;
            for (int k = 0; k <= K; ++k) o.out_tok[(int64_t)b * (K + 1) + k] = -1;
            o.seq_status[b] |= TLI_FLAG_NONFINITE;
        } else {
            o.out_tok[(int64_t)b * (K + 1) + f.n] = r.tok;
            if (f.bonus && o.lse_p) o.lse_p[(int64_t)b * (K + 1) + K] = r.lse_bonus;
            if (r.add_flags) o.seq_status[b] |= r.add_flags;
        }
    }
}

// ---- kernel: chunk masses of the row the extra token is drawn from ------------------------------
// Residual rows (first rejection at position n < K).  The extra token is drawn from
// r(t) ∝ max(0, p_n(t) - q'_n(t)), and per chunk of target ids
//     sum_chunk max(0, p - q') = sum_chunk p - sum_{shared ids of the chunk} min(p, q').
// The first sum is known: the normaliser kernel left the chunk table (ref, s) of every target row, and
// sum_chunk p = s * 2^(ref * c_true/c - lse_p * log2 e).  Only the second sum is computed here; it runs over
// the shared PAIRS (target id, drafter id) alone.  The two vocabularies' orders are unrelated, so a pair
// needs one random access on each side -- and random access is cheap only in LDS.  The target row is cut
// into PARTS, runs of whole chunks holding at most part_cap pairs.  A workgroup owns one part of one row.
//   (1) It sweeps the drafter row with plain 16-byte loads and packs the logits of the part's pairs into LDS in
//       ascending drafter order.  Beside every vector of the row the map holds one word: which of the vector's
//       elements belong to the part, and the LDS position of the first of them.  A lane stores all its
//       elements, the unwanted ones to a scratch word of its own, so the sweep has no branch, no mask
//       juggling and no index list.  (Gathering the part through an index list was tried first: a 2-byte
//       gather costs the texture addresser ~30 cycles per wave instruction, more than the whole target row.)
//   (2) Its waves stream the part's target chunks: a wave parks a chunk in its private LDS slot and walks the
//       map's list of the chunk's pairs, each entry = (byte offset in chunk, index of the staged drafter
//       logit), reading both logits from LDS.
// Every target chunk is thus read once per row, every pair is owned by one lane of one wave, and sums are
// per lane, then across lanes in a fixed order, so results do not depend on timing.
// The kernel is short (tens of microseconds) and its waves are few (16 per CU): counters show it bound by
// instruction issue and by dependent round trips, not by bandwidth.  Hence:
//   * a chunk's pair list is padded to whole groups of 128 entries (two per lane, one 8-byte load) with
//     entries that point at a -inf logit (min(p, 0) contributes exactly 0): a group is either all live or
//     absent and the only test is a wave-uniform one; the list has kPairU groups of slack at its end, so the
//     first kPairU groups of every chunk are fetched without looking at its length;
//   * an entry is two 16-bit fields that the address arithmetic reads in place;
//   * the loads of a wave's next chunk are in flight while it works on the current one (two register sets,
//     alternating), those of its first chunk are issued before the staging sweep, and the list bounds of
//     all its chunks come with one vector load (scalar loads would miss the scalar cache at every step, and
//     a wait for one of them is a wait for everything else the wave has in flight on that counter);
//   * no load sits under a branch (the compiler would then wait for ALL outstanding loads at every use): a
//     fetch past the end of the part is made harmless, every lane reading the same few lines again.
// Output: mn[b][chunk] = sum of min(p, q') over the chunk's pairs; the draw kernel forms the masses.
// Bonus rows (nothing rejected) go through the same grid: the workgroups of a sequence split target row K
// and scan it into a plain (ref, s) softmax table.
// grid (B rounded up to 8) x nparts x nsplit; workgroups of flagged sequences exit at once.
// nsplit > 1 (few sequences): the chunks of one (sequence, part) are dealt to nsplit workgroups, each with
// its own copy of the part's drafter logits.
constexpr int kStageV = 8;             // drafter vectors a lane has in flight during the staging sweep
constexpr float kPreciseBelow = 0.1f;  // see precise_chunk_masses

struct ScanLists {            // the map's lists for one dtype and one drafter-row layout, as the scan kernel reads them
    int nparts;
    int row_elems;            // valid entries of a drafter row: |D| (full layout) or |T∩D| (compact)
    int NV;                   // vectors of a drafter row, rounded up to whole groups of 64
    const int32_t* cb;        // [nparts+1] first chunk of every part
    const int32_t* part_n;    // [nparts] pairs of every part
    const int2* grange;       // [nparts] first and one-past-last group of 64 vectors that hold a logit of the part
    const uint32_t* stab;     // [nparts][NV] per vector: staged index of its first logit of the part | which of its
                              //     elements belong to the part << 16
    const int32_t* pl_g;      // [nC+1] first group of every chunk's pair list
    const uint2* pl_e;        // pairs grouped by chunk (two per lane and group), kPairU groups of slack at the end
};
// NaN or +inf among the staged drafter logits must surface (-inf is legal).  As signed integers the raw
// patterns of +inf and the positive NaNs are the largest values, as unsigned ones the negative NaNs are (just
// above -inf): two running maxima, taken on both halves of a dword at once for bf16.
template <int DT> struct BadTrack;
template <> struct BadTrack<TLI_BF16> {
    typedef short s2v __attribute__((ext_vector_type(2)));
    typedef unsigned short us2v __attribute__((ext_vector_type(2)));
    s2v sm = {(short)-32768, (short)-32768};
    us2v um = {0, 0};
    __device__ __forceinline__ void add(uint32_t w) {
        sm = __builtin_elementwise_max(sm, __builtin_bit_cast(s2v, w));
        um = __builtin_elementwise_max(um, __builtin_bit_cast(us2v, w));
    }
    __device__ __forceinline__ void add_one(uint32_t raw) { add(raw | (raw << 16)); }
    __device__ __forceinline__ bool bad() const {
        return sm.x >= (short)0x7f80 || sm.y >= (short)0x7f80 || um.x > 0xff80u || um.y > 0xff80u;
    }
};
template <> struct BadTrack<TLI_F32> {
    int32_t sm = INT32_MIN;
    uint32_t um = 0;
    __device__ __forceinline__ void add(uint32_t w) {
        sm = max(sm, (int32_t)w);
        um = max(um, w);
    }
    __device__ __forceinline__ void add_one(uint32_t raw) { add(raw); }
    __device__ __forceinline__ bool bad() const { return sm >= 0x7f800000 || um > 0xff800000u; }
};

// Residual masses of a workgroup's target chunks for a row on which the two models nearly agree.  The fast walk
// forms a chunk's mass as (sum of p over the chunk, from the normaliser kernel) - (sum of min(p, q') over its pairs):
// two fp32 sums, each good to 1e-7 of the chunk's p mass, so their difference is only that good -- and the draw
// needs the row's masses to 1e-6 of the ROW's residual mass R.  All the p mass of a row is one, so with a tenth of
// it residual (and a workgroup's own chunks are a part of the row's) the fast masses will do whatever they are; and a
// chunk whose own residual is a tenth or more of its p mass is good to 1e-6 of itself.  The other chunks of a
// workgroup that cannot see that tenth are formed again here, with nothing subtracted that does not cancel exactly:
//     mass = (sum over every id of the chunk of p  -  sum over the pairs of p)  +  sum over the pairs of max(0, p - q'),
// all three in fp64 over fp32 terms, p of a shared id being the same fp32 number in both sums (same instructions, same
// operands), so the first difference is the target-only ids' mass to fp64 rounding; the last sum takes its terms from
// residual_weight.  Padding entries of a pair list (first id of the chunk against a -inf drafter logit) add the same p
// to the second and the third sum.  The chunk's mass goes to rmass, where the fast walk's would have gone.
template <int DT>
__device__ __noinline__ void precise_chunk_masses(unsigned char* lds, uint32_t tb, const char* trow, int nvec, int Vt,
                                                  const int32_t* pl_g, const uint2* pl_e, int c_lo,
                                                  const uint16_t* list, int n_list, int w, int nw, ResidualParams rp,
                                                  double l2p, double* rmass_row) {
    constexpr int EPV = Traits<DT>::EPV;
    constexpr int ESZ = Traits<DT>::ESZ;
    typedef typename std::conditional<DT == TLI_BF16, uint16_t, uint32_t>::type raw_t;
    const int lane = threadIdx.x & 63;
    unsigned char* const part = lds + kTrashBytes;
    const ResidualWide rw = widen(rp, l2p);
    // the workgroup's list of chunks is dealt to its waves in turn: whoever owned a chunk in the walk, the heavy
    // ones are spread evenly now
    for (int i = w; i < n_list; i += nw) {  // wave-uniform
        const int c = c_lo + (int)list[i];
        const uint32_t v0 = (uint32_t)c * (kLoads * kWave) + lane;
        u4v v[kLoads];
#pragma unroll
        for (int j = 0; j < kLoads; ++j)
            v[j] = *reinterpret_cast<const u4v*>(trow + min(v0 + j * kWave, (uint32_t)nvec - 1u) * 16u);
        // the head of the chunk's pair list with them (the list is padded: reading kPairU groups is always in bounds)
        const int g0 = pl_g[c], g1 = pl_g[c + 1];
        uint2 eh[kPairU];
#pragma unroll
        for (int k2 = 0; k2 < kPairU; ++k2) eh[k2] = pl_e[(int64_t)(g0 + k2) * kWave + lane];
        u4v* st = reinterpret_cast<u4v*>(lds + tb);
#pragma unroll
        for (int j = 0; j < kLoads; ++j) st[j * kWave + lane] = v[j];
        __builtin_amdgcn_wave_barrier();
        double s_all = 0.0, s_pairs = 0.0, s_w = 0.0;
#pragma unroll
        for (int j = 0; j < kLoads; ++j) {
            float x[EPV];
            unpack<DT>(to_uint4(v[j]), x);
            const int64_t e0 = (int64_t)(v0 + j * kWave) * EPV;
#pragma unroll
            for (int i = 0; i < EPV; ++i) {
                const float pi = exp2_split(x[i], rp.ct_hi, rp.ct_lo, rp.lp_hi, rp.lp_lo);
                s_all += (e0 + i < Vt) ? (double)pi : 0.0;
            }
        }
        auto one = [&](uint32_t e) {
            const uint32_t xr = *reinterpret_cast<const raw_t*>(lds + (tb + (e & 0xffffu)));
            const uint32_t yr = *reinterpret_cast<const raw_t*>(part + (e >> kPairShift) * ESZ);
            const float xv = as_f(DT == TLI_BF16 ? xr << 16 : xr), yv = as_f(DT == TLI_BF16 ? yr << 16 : yr);
            const float pi = exp2_split(xv, rp.ct_hi, rp.ct_lo, rp.lp_hi, rp.lp_lo);
            s_pairs += (double)pi;
            s_w += residual_weight(pi, xv, yv, rw);
        };
#pragma unroll
        for (int k2 = 0; k2 < kPairU; ++k2)
            if (g0 + k2 < g1) { one(eh[k2].x); one(eh[k2].y); }  // wave-uniform test
        for (int g = g0 + kPairU; g < g1; ++g) {
            const uint2 e = pl_e[(int64_t)g * kWave + lane];
            one(e.x);
            one(e.y);
        }
        __builtin_amdgcn_wave_barrier();  // the slot is rewritten by the next chunk
        const double mass = (wave_sum_f64(s_all) - wave_sum_f64(s_pairs)) + wave_sum_f64(s_w);
        if (lane == 0) rmass_row[c] = mass > 0.0 ? mass : (mass != mass ? mass : 0.0);
    }
}

// DIAG (acceptance-rate diagnostics): the items are all B*K positions instead of one row per sequence, and a
// second sum runs beside the first with the drafter's unrestricted probabilities q = q' * 2^-dq:
// mn = sum min(p, q') (TLI's expected acceptance rate), mn2 = sum min(p, q) (the union algorithm's).
// MODE 2 is the same diagnostic scan with the exponent arguments in fp64 and every term scaled by an exact power of
// two: for the positions marked in `redo`, whose rates came out so small in MODE 1 that the fp32 arguments (good to
// 2^-24 of their magnitude, i.e. 5e-6 of a term at 2^-100) and the fp32 range (nothing below 2^-126) show.
// ACCEPT (MODE 0 only; small batches, which keep the split form): the sequence's record is not read from `frow` but
// formed here -- wave 0 of every workgroup of the sequence runs accept_sequence and hands the record to the other
// waves through LDS; the sequence's first workgroup stores the outputs.  A kernel launch and its start-up less.
template <int DT, int MODE, bool ACCEPT = false>
__global__ __launch_bounds__(kScanWG) void k_final_scan(
    const void* __restrict__ logits_t, DrafterView dv, int B, int K, int Vt, int Vd, int nC, int nsplit, ScanLists ls,
    float cs_t, double ratio_t, const FinalRow* __restrict__ frow, float* __restrict__ tab_ref, float* __restrict__ tab_s, double* __restrict__ mn, double* __restrict__ mn2,
    int32_t* __restrict__ fbad, const int32_t* __restrict__ redo, const float2* __restrict__ ctab,
    double* __restrict__ rmass, AcceptIn ain = AcceptIn(), AcceptOut aout = AcceptOut()) {
    constexpr bool DIAG = MODE != 0;
    constexpr bool EXACT = MODE == 2;
    constexpr int EPV = Traits<DT>::EPV;
    constexpr int ESZ = Traits<DT>::ESZ;
    typedef typename std::conditional<DT == TLI_BF16, uint16_t, uint32_t>::type raw_t;
    __shared__ __attribute__((aligned(16))) unsigned char lds[kScanLds];
    unsigned char* const part = lds + kTrashBytes;  // staged logit i at part + i * ESZ
    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  The workgroups of one sequence
    // stream the same rows, so they are given ids that land on the same XCD, next to each other in time:
    // id = slot * 8 + xcd, sequence = (slot / per_seq) * 8 + xcd, (part, split) = slot % per_seq.
    const int nparts = ls.nparts;
    const int per_seq = nparts * nsplit;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int b = (slot / per_seq) * 8 + xcd, sub = slot % per_seq;
    const int p = sub / nsplit, sp = sub - p * nsplit;
    if (b >= B) return;
    // What the part is and where the lists of this wave's chunks begin do not depend on the sequence: they are
    // fetched beside the sequence's record rather than after it.
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int c_lo = ls.cb[p], c_hi = ls.cb[p + 1];
    const int2 gr = ls.grange[p];
    const int ns = ls.part_n[p];
    const int ncp = c_hi - c_lo;  // 1 .. kMaxPartChunks
    const int gw = sp * kScanWaves + wave, stride = nsplit * kScanWaves;  // this wave takes chunks gw, gw + stride, ...
    const int32_t* __restrict__ pl_g = ls.pl_g;
    const uint2* __restrict__ pl_e = ls.pl_e;
    // The list bounds (in groups of kPairG entries) of the wave's chunks: lane k holds those of its k-th chunk,
    // lanes past the wave's last chunk those of the part's first chunk.
    int2 gbv;
    {
        const int idx = gw + lane * stride;
        const int c = c_lo + (idx < ncp ? idx : 0);
        gbv = make_int2(pl_g[c], pl_g[c + 1]);
    }
    if (EXACT && !redo[b]) return;
    __shared__ FinalRow s_frow;
    if (ACCEPT) {
        if (wave == 0) {
            const FinalRow mine = accept_sequence<DT>(b, logits_t, dv, K, Vt, Vd, ain, aout, sub == 0);
            if (lane == 0) s_frow = mine;
        }
        __syncthreads();
    }
    const FinalRow f = ACCEPT ? s_frow : frow[b];
    if (f.skip) return;
    if (f.bonus) {
        const u4v* rowk = reinterpret_cast<const u4v*>(static_cast<const char*>(logits_t) + (int64_t)f.t_row * Vt * ESZ);
        float* br = tab_ref + (int64_t)b * nC;
        float* bs = tab_s + (int64_t)b * nC;
        const int cps = (nC + per_seq - 1) / per_seq;
        scan_chunks<DT, false, kScanWaves>(rowk, Vt, min(nC, sub * cps), min(nC, (sub + 1) * cps), cs_t,
                                           (float)(ratio_t - 1.0), nullptr, [&](int c, float r, float sc) {
                                               if (lane == 0) { br[c] = r; bs[c] = sc; }
                                           });
        return;
    }
    if (!f.rp.use_q) return;  // q' = 0 everywhere: the masses are the chunk sums of p, nothing to subtract
    // rows as byte pointers: every offset below fits 32 bits, which keeps the address arithmetic to one instruction
    const char* __restrict__ drow = static_cast<const char*>(dv.base) + (int64_t)f.d_row * dv.row_stride * ESZ;
    const char* __restrict__ trow = static_cast<const char*>(logits_t) + (int64_t)f.t_row * Vt * ESZ;
    const int nvec = (Vt + EPV - 1) / EPV;

    struct Fetched {
        u4v v[kLoads];
        uint2 e[kPairU];
    };
    // Loads of the wave's chunk number k and of the head of its pair list.  Past the end of the part every lane
    // reads lane 0's addresses of the part's first chunk: a few cache lines, nothing new.
    auto fetch = [&](int k, Fetched& r) {
        const int idx = gw + k * stride;
        const bool ok = idx < ncp;
        const int c = c_lo + (ok ? idx : 0);
        const uint32_t ln = ok ? lane : 0;
        const uint32_t g0 = __builtin_amdgcn_readlane(gbv.x, k);
        const uint32_t v0 = (uint32_t)c * (kLoads * kWave) + ln;
#pragma unroll
        // (vectors past the row's end re-read its last vector: no pair points there.  A target chunk is read once:
        // non-temporal, 4 us off the kernel on rows that come from HBM -- 45.6 against 49.6 us -- while the drafter
        // row, which the row's other part sweeps again, is better left to the caches: 48.2 us with both.)
        for (int j = 0; j < kLoads; ++j)
            r.v[j] = __builtin_nontemporal_load(reinterpret_cast<const u4v*>(trow + min(v0 + j * kWave, (uint32_t)nvec - 1u) * 16u));
        const char* ep = reinterpret_cast<const char*>(pl_e) + (size_t)g0 * (kWave * 8);
#pragma unroll
        for (int k2 = 0; k2 < kPairU; ++k2) r.e[k2] = *reinterpret_cast<const uint2*>(ep + (ln * 8u + k2 * (kWave * 8)));
    };
    Fetched fa, fb;
    fetch(0, fa);

    // ---- (1) the drafter logits of this part's pairs -> LDS
    {
        const int nvd = (ls.row_elems + EPV - 1) / EPV;
        // The part's groups of 64 vectors are dealt to the waves in equal runs.  (The waves of a workgroup do not
        // start together: they are launched four at a time, the last four some 17,000 cycles after the first.
        // Giving the early ones more of the sweep was tried and moved the barrier by little: the late waves'
        // own first round trips to memory are what it waits for.)
        const int per_wave = (gr.y - gr.x + kScanWaves - 1) / kScanWaves;
        const int gbeg = gr.x + wave * per_wave, gend = min(gbeg + per_wave, gr.y);
        if (tid == 0)
            *reinterpret_cast<uint32_t*>(part + dummy_index<DT>() * ESZ) = DT == TLI_BF16 ? 0xff80ff80u : 0xff800000u;
        const uint32_t mine = (uint32_t)lane * 4;  // the lane's scratch word
        const char* __restrict__ stab = reinterpret_cast<const char*>(ls.stab + (int64_t)p * ls.NV);
        const uint32_t vlast = (uint32_t)min(gend * kWave, nvd) - 1u;  // the wave's last vector
        for (int g0 = gbeg; g0 < gend; g0 += kStageV) {  // wave-uniform
            u4v v[kStageV];
            uint32_t tv[kStageV];
#pragma unroll
            for (int u = 0; u < kStageV; ++u) {
                // past the wave's last vector: that vector is done again, the same bytes to the same places
                const uint32_t vi = min((uint32_t)(g0 + u) * kWave + lane, vlast);
                v[u] = *reinterpret_cast<const u4v*>(drow + vi * 16u);
                tv[u] = *reinterpret_cast<const uint32_t*>(stab + vi * 4u);
            }
#pragma unroll
            for (int u = 0; u < kStageV; ++u) {
                const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
                // d = (LDS address of the lane's next kept logit) - mine, so address = mine + keep * d
                uint32_t d = kTrashBytes + (tv[u] & 0xffffu) * ESZ - mine;
#pragma unroll
                for (int i = 0; i < EPV; ++i) {
                    const uint32_t k1 = (tv[u] >> (16 + i)) & 1u;
                    uint32_t at;  // = mine + k1 * d (d < 2^24; written out because the compiler would mask d first)
                    asm("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(at) : "v"(k1), "v"(d), "v"(mine));
                    if (DT == TLI_BF16)
                        *reinterpret_cast<uint16_t*>(lds + at) = (uint16_t)(i & 1 ? w[i >> 1] >> 16 : w[i >> 1]);
                    else
                        *reinterpret_cast<uint32_t*>(lds + at) = w[i];
                    // d += k1 * ESZ, likewise (the compiler would keep a count and rebuild d from it, an instruction more)
                    asm("v_lshl_add_u32 %0, %1, %2, %0" : "+v"(d) : "v"(k1), "n"(ESZ == 2 ? 1 : 2));
                }
            }
        }
    }
    __syncthreads();

    // NaN / +inf among the staged logits (the flag is stored at the very end: a pending store would turn every
    // wait for a load into a wait for all of them)
    BadTrack<DT> bt;
    {
        const int nfull = ns / EPV;
        const uint4* lv = reinterpret_cast<const uint4*>(part);
        for (int o = tid; o < nfull; o += kScanWG) {
            const uint4 w = lv[o];
            bt.add(w.x); bt.add(w.y); bt.add(w.z); bt.add(w.w);
        }
        if (tid < ns - nfull * EPV) bt.add_one(reinterpret_cast<const raw_t*>(part)[nfull * EPV + tid]);
    }

    // ---- (2) stream target chunks past it
    double* my_mn = DIAG ? mn + (int64_t)b * nC : nullptr;
    double* my_mn2 = DIAG ? mn2 + (int64_t)b * nC : nullptr;
    const ResidualParams rp = f.rp;
    const uint32_t tb = (uint32_t)(kPartBytes + wave * kSlotBytes);
    // log2 p = x*ct - Lp and log2 q' = y*cd - Lq in two-term form.  The subtrahends are pinned to vector registers:
    // an instruction may read one scalar register only, and the compiler would otherwise copy them over per use.
    float nlp_hi = -rp.lp_hi, nlp_lo = -rp.lp_lo, nlq_hi = -rp.lq_hi, nlq_lo = -rp.lq_lo;
    asm volatile("" : "+v"(nlp_hi), "+v"(nlp_lo), "+v"(nlq_hi), "+v"(nlq_lo));
    // min(p, q') of one pair = 2^min(log2 p, log2 q'): one exponential per pair
    const float dq = f.dq;
    auto pair_min = [&](uint32_t e, float& second) -> float {
        const uint32_t xr = *reinterpret_cast<const raw_t*>(lds + (tb + (e & 0xffffu)));
        const uint32_t yr = *reinterpret_cast<const raw_t*>(part + (e >> kPairShift) * ESZ);
        const float xv = as_f(DT == TLI_BF16 ? xr << 16 : xr), yv = as_f(DT == TLI_BF16 ? yr << 16 : yr);
        const float a = fmaf(xv, rp.ct_hi, nlp_hi) + fmaf(xv, rp.ct_lo, nlp_lo);
        const float bq = fmaf(yv, rp.cd_hi, nlq_hi) + fmaf(yv, rp.cd_lo, nlq_lo);
        if (DIAG) second = exp2_hw(fminf(a, bq - dq));
        return exp2_hw(fminf(a, bq));
    };
    // MODE 2: log2 p and log2 q' in fp64, a term = 2^fraction (the hardware exponential on an argument in
    // [-0.5, 0.5]) times an exact power of two, in fp64: good to the exponential's 1e-7 at any size
    const double ct64 = (double)rp.ct_hi + (double)rp.ct_lo, cd64 = (double)rp.cd_hi + (double)rp.cd_lo;
    const double lq64 = (double)rp.lq_hi + (double)rp.lq_lo;
    const double dq64 = (double)f.dq + (double)f.dq_lo;
    auto exp2_wide = [](double m) -> double {
        if (!(m > -1070.0)) return m != m ? m : 0.0;  // -inf, or below what fp64 holds (NaN stays NaN)
        const double n = rint(m);
        return ldexp((double)exp2_hw((float)(m - n)), (int)n);
    };
    auto pair_min_wide = [&](uint32_t e, double& second) -> double {
        const uint32_t xr = *reinterpret_cast<const raw_t*>(lds + (tb + (e & 0xffffu)));
        const uint32_t yr = *reinterpret_cast<const raw_t*>(part + (e >> kPairShift) * ESZ);
        const float xv = as_f(DT == TLI_BF16 ? xr << 16 : xr), yv = as_f(DT == TLI_BF16 ? yr << 16 : yr);
        const double a = fma((double)xv, ct64, -f.l2p), bq = fma((double)yv, cd64, -lq64);
        second = exp2_wide(fmin(a, bq - dq64));
        return exp2_wide(fmin(a, bq));
    };
    // Results stay in registers until the wave is through (lane k keeps the sum of the wave's k-th chunk):
    // a store shares the loads' completion counter and completes out of order with them, so while one may
    // be pending every wait for a load degrades to a wait for all loads.
    double keep = 0.0, keep2 = 0.0;
    auto process = [&](const Fetched& r, int k) {
        u4v* st = reinterpret_cast<u4v*>(lds + tb);
#pragma unroll
        for (int j = 0; j < kLoads; ++j) st[j * kWave + lane] = r.v[j];
        // one wave writes and reads its slot: its LDS operations execute in order and the compiler keeps
        // may-alias accesses in program order; the wave barrier only pins the schedule
        __builtin_amdgcn_wave_barrier();
        float acc = 0.f, acc2 = 0.f;
        double wacc = 0.0, wacc2 = 0.0;
        auto two = [&](uint2 e) {
            if (EXACT) {
                double u0, u1;
                const double t0 = pair_min_wide(e.x, u0), t1 = pair_min_wide(e.y, u1);
                wacc += t0 + t1;
                wacc2 += u0 + u1;
            } else {
                float u0 = 0.f, u1 = 0.f;
                const float t0 = pair_min(e.x, u0), t1 = pair_min(e.y, u1);
                acc += t0 + t1;
                if (DIAG) acc2 += u0 + u1;
            }
        };
        const int g0 = __builtin_amdgcn_readlane(gbv.x, k), g1 = __builtin_amdgcn_readlane(gbv.y, k);
        const int ng = g1 - g0;
#pragma unroll
        for (int k2 = 0; k2 < kPairU; ++k2)
            if (k2 < ng) two(r.e[k2]);  // wave-uniform test
        for (int g = g0 + kPairU; g < g1; ++g) two(pl_e[(int64_t)g * kWave + lane]);  // crowded chunk: the rest
        __builtin_amdgcn_wave_barrier();  // the slot is rewritten by the next chunk
        // A chunk's sum is taken in fp32: a lane's dozen-odd terms in turn, the 64 lane totals on the DPP network
        // (one instruction per step; a double takes five).  That is a relative 1e-7, the size of the exponential's
        // own error; chunk sums are combined in fp64 downstream.
        if (EXACT) {
            const double tot = wave_sum_f64(wacc), tot2 = wave_sum_f64(wacc2);
            if (lane == k) { keep = tot; keep2 = tot2; }
        } else {
            const float tot = wave_sum(acc);
            if (lane == k) keep = (double)tot;
            if (DIAG) {
                const float tot2 = wave_sum(acc2);
                if (lane == k) keep2 = (double)tot2;
            }
        }
    };
    // (for the question asked after the walk: the p mass of the wave's chunks, lane k the k-th; loaded here so that
    // the answer does not wait for memory)
    float2 my_rs = make_float2(-INFINITY, 0.f);
    if (MODE == 0) {
        const int idx = gw + lane * stride;
        if (idx < ncp) my_rs = ctab[(int64_t)f.d_row * nC + c_lo + idx];
    }
    int k = 0;
    for (int idx = gw; idx < ncp; idx += 2 * stride, k += 2) {
        fetch(k + 1, fb);
        process(fa, k);
        fetch(k + 2, fa);
        if (idx + stride < ncp) process(fb, k + 1);
    }
    __shared__ uint16_t again_list[kMaxPartChunks];  // the workgroup's chunks that are formed again in the precise form
    __shared__ int again_n;                          // (as offsets from c_lo)
    if (MODE == 0 && tid == 0) again_n = 0;  // (a barrier lies between this and the first append)
    const int my_idx = gw + lane * stride;  // lane k: the wave's k-th chunk
    if (DIAG) {
        if (my_idx < ncp) { my_mn[c_lo + my_idx] = keep; my_mn2[c_lo + my_idx] = keep2; }
    } else {
        double mass_fast = 0.0, my_p = 0.0;
        float pm = 0.f, rm = 0.f;  // rough figures are all the questions below need
        if (my_idx < ncp) {
            // the chunk's mass as the draw takes it: sum_chunk p (the normaliser kernel's pair) - sum of min(p, q')
            my_p = (my_rs.x == -INFINITY) ? 0.0 : (double)my_rs.y * exp2((double)my_rs.x * ratio_t - f.l2p);
            const double t = my_p - keep;
            mass_fast = t > 0.0 ? t : (t != t ? t : 0.0);
            pm = (float)my_p;
            rm = (float)mass_fast;
        }
        pm = wave_sum(pm);
        rm = wave_sum(rm);
        float* dec = reinterpret_cast<float*>(lds);  // the sweep's scratch words: free since the barrier behind it
        if (lane == 0) { dec[2 * wave] = pm; dec[2 * wave + 1] = rm; }
        __syncthreads();
        float P = 0.f, R = 0.f;  // the workgroup's p mass and residual mass (the same in every wave)
#pragma unroll
        for (int w = 0; w < kScanWaves; ++w) { P += dec[2 * w]; R += dec[2 * w + 1]; }
        // Which chunks need the precise form (see precise_chunk_masses)?  None if the workgroup's chunks hold a tenth
        // of the row's p mass (one) as residual, or a quarter of their own (their errors then add up to 4e-7 of it).
        // Else those that hold less than a tenth of their own p mass as residual -- but not the light ones: the chunks
        // with less p mass than their even share of 2.5 R add up to 2.5e-7 of R between them (R less what the fast
        // sums themselves may have added to it).  NaN sums ask for nothing: the draw reports those.
        const bool some = R < kPreciseBelow && R < 0.25f * P;
        const double light = 2.5 * (double)fmaxf(R - 2e-7f * P, 0.f) / (double)ncp;
        const bool again = some && my_idx < ncp && mass_fast < (double)kPreciseBelow * my_p && my_p > light;
        if (my_idx < ncp && !again) rmass[(int64_t)b * nC + c_lo + my_idx] = mass_fast;
        if (some) {  // (uniform over the workgroup: every wave meets at this barrier or none does)
            if (again) again_list[atomicAdd(&again_n, 1)] = (uint16_t)my_idx;
            __syncthreads();
            precise_chunk_masses<DT>(lds, tb, trow, nvec, Vt, pl_g, pl_e, c_lo, again_list, again_n, wave, kScanWaves, rp,
                                     f.l2p, rmass + (int64_t)b * nC);
        }
    }
    if (bt.bad()) fbad[b] = 1;
}

// kernel: draw the extra token of every sequence from its row's chunk tables.  grid (B), kLoads waves: every wave
// finds the chunk for itself (the tables are small and shared), then each takes a quarter of the chunk.
template <int DT>
__global__ __launch_bounds__(kLoads * kWave) void k_final_pick(const void* __restrict__ logits_t, DrafterView dv,
                                                       int K, int Vt, int Vd, int nC, float cs_t, double ratio_t,
                                                       const FinalRow* __restrict__ frow,
                                                       const int32_t* __restrict__ t2d,
                                                       const float* __restrict__ tab_ref,
                                                       const float* __restrict__ tab_s,
                                                       const float2* __restrict__ ctab,
                                                       const double* __restrict__ rmass,
                                                       const int32_t* __restrict__ fbad, FinalOut o) {
    const int b = blockIdx.x;
    // the chunk masses do not wait for the sequence's record: both round trips are started together (for rows that
    // have none the words read here are never looked at)
    __shared__ double s_mass[kLdsChunks];
    const bool staged = nC <= kLdsChunks;
    if (staged)
        for (int c = threadIdx.x; c < nC; c += kLoads * kWave) s_mass[c] = rmass[(int64_t)b * nC + c];
    const int bad = fbad[b];
    const FinalRow f = frow[b];
    __syncthreads();
    if (f.skip) return;
    final_pick_row<DT>(f, b, logits_t, dv, K, Vt, Vd, nC, cs_t, ratio_t, t2d, tab_ref + (int64_t)b * nC,
                       tab_s + (int64_t)b * nC, ctab, staged ? s_mass : rmass + (int64_t)b * nC, f.rp.use_q && bad != 0, o);
}
