// tli_seq_kernels.h -- Normalisers and accept tests of a sequence in one persistent workgroup (batches of about one sequence per
// compute unit and more).  Included by tli_kernels.hip inside its unnamed namespace, after tli_verify_kernels.h.
#pragma once

// Standard SD appendix, verification loop and count of accepted drafts, in one kernel (k_lse + the accept tests of the
// split form, without a kernel boundary between the normalisers and the tests).  A workgroup of
// 1 + kSeqStreamWaves waves owns a sequence:
//   * waves 1.. stream the sequence's K target rows, one row at a time, chunk pairs (ref, s) into one of two
//     tables in LDS, rows in position order (on rows that come from HBM this beats reversed and per-sequence
//     rotated orders by 2.5 us: 212.3 against 214.8 us for the call);
//   * wave 0 is the sequence's clerk: while the others stream the next row it reduces the last row's pairs to the
//     row's log-normaliser (and leaves the pairs in ctab for the residual step), and lane k takes position k's
//     accept test the moment row k is through -- its draft's two logits were gathered when the kernel started;
//   * when every row is through the clerk runs the first-reject scan and writes the sequence's outputs and the
//     record the extra-token kernels start from, exactly as accept_sequence does.
// The chunk loop is k_lse's.  Eight streaming waves per compute unit (64 KB of loads in flight each, 16 MB over the
// chip) is where the rate peaks: 153-156 us for the large-vocabulary batch's 1.05 GB against 157 us with 10 to 15
// waves, 163 with 6, 180 with 4 or 5 -- and against 175 / 188 us with two / three chunks in flight per wave instead of one.
// Requires nC <= kSeqMaxChunks; grid (B), kSeqWG threads.
constexpr int kSeqMaxChunks = 1024;  // chunks of a target row: two tables of pairs in LDS
constexpr int kSeqStreamWaves = 8;
constexpr int kSeqWG = (1 + kSeqStreamWaves) * kWave;

struct SeqIn {
    const int32_t *d2t, *tok_d;
    const double* lse_q;
    const float* u_acc;
    double ratio_t, inv_temp_t, inv_temp_d, c_t, c_d;
    float cs_t;
    int union_mode;
};
struct SeqOut {
    int32_t *n_accepted, *out_tok;
    uint8_t* accept;
    double *p_tok, *q_tok, *lse_p;
    int32_t* seq_status;
    FinalRow* frow;
    int32_t* fbad;
};

template <int DT>
__global__ __launch_bounds__(kSeqWG) void k_lse_accept_seq(const void* __restrict__ logits_t, DrafterView dv, int K,
                                                            int Vt, int Vd, int nC, SeqIn in, float2* __restrict__ ctab,
                                                            SeqOut out) {
    constexpr int ESZ = Traits<DT>::ESZ;
    __shared__ float2 stash[2 * kSeqMaxChunks];
    const int b = blockIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const double kd = (in.ratio_t - 1.0) * kLn2;

    // ---- the clerk's state: lane k = position k
    bool bad = false, acc = false, nonfinite = false;
    int tt = -1;
    float xt = 0.f, xd = 0.f, my_u = 0.f;
    double my_lq = 0.0, my_lse = 0.0;
    if (wave == 0 && lane < K) {
        const int64_t row = (int64_t)b * K + lane;
        const int d = in.tok_d[row];
        my_lq = in.lse_q[row];
        my_u = in.u_acc[row];
        // TLI: a draft must be a shared drafter id.  Union algorithm: any drafter id is a legal draft (see accept_sequence).
        if (d < 0 || d >= Vd || (!in.union_mode && in.d2t[d] < 0)) {
            bad = true;
        } else {
            tt = in.d2t[d];
            const char* lt = static_cast<const char*>(logits_t) + ((int64_t)b * (K + 1) + lane) * Vt * ESZ;
            const char* ld = static_cast<const char*>(dv.base) + row * dv.row_stride * ESZ;
            if (tt >= 0) xt = load_elem<DT>(lt, tt);
            xd = load_elem<DT>(ld, dv.d2x ? dv.d2x[d] : d);
        }
    }

    for (int i = 0; i <= K; ++i) {
        if (i < K && wave != 0) {  // streaming waves: row i -> table i & 1; chunk c by wave 1 + c % 8
            const int k = i;
            const u4v* rowv = reinterpret_cast<const u4v*>(static_cast<const char*>(logits_t) +
                                                            ((int64_t)b * (K + 1) + k) * Vt * ESZ);
            float2* buf = stash + (i & 1) * kSeqMaxChunks;
            // (first chunk -1: the scan gives wave w the chunks first + w, first + w + 8, ...)
            scan_chunks<DT, false, kSeqStreamWaves>(rowv, Vt, -1, nC, in.cs_t, (float)(in.ratio_t - 1.0), nullptr,
                                                   [&](int c, float r, float sc) {
                                                       if (lane == 0) buf[c] = make_float2(r, sc);
                                                   });
        }
        if (i > 0 && wave == 0) {  // the clerk: row i - 1 from table (i - 1) & 1
            const int k = i - 1;
            const int64_t row = (int64_t)b * K + k;
            const float2* buf = stash + ((i - 1) & 1) * kSeqMaxChunks;
            float r_mine = -INFINITY;
            for (int c = lane; c < nC; c += kWave) {
                const float2 e = buf[c];
                r_mine = fmaxf(r_mine, e.x);
                ctab[row * nC + c] = e;  // the residual's chunk sums of p come from here
            }
            const float R = wave_max(r_mine);
            double s_mine = 0.0;
            for (int c = lane; c < nC; c += kWave) {
                const float2 e = buf[c];
                s_mine += (double)e.y * exp2_diff(e.x, R, kd);
            }
            const double S = wave_sum_f64(s_mine);
            double lse;  // as combine_parts
            if (S != S || R == INFINITY) lse = NAN;
            else if (!(S > 0.0)) lse = -INFINITY;
            else lse = kLn2 * ((double)R * in.ratio_t + log2(S));
            if (lane == k) {
                my_lse = lse;
                nonfinite = lse != lse;
                double pd = 0.0, qd = 0.0;
                if (bad) {
                } else if (in.union_mode && my_lq != my_lq) {
                    nonfinite = true;
                } else if (!nonfinite) {
                    pd = (tt < 0 || lse == -INFINITY) ? 0.0 : exp((double)xt * in.inv_temp_t - lse);
                    qd = (in.union_mode && my_lq == -INFINITY) ? 0.0 : exp((double)xd * in.inv_temp_d - my_lq);
                    acc = (double)my_u * qd < pd;
                }
                if (out.accept) out.accept[row] = acc ? 1 : 0;
                if (out.p_tok) out.p_tok[row] = pd;
                if (out.q_tok) out.q_tok[row] = qd;
                if (out.lse_p) out.lse_p[(int64_t)b * (K + 1) + k] = lse;
            }
        }
        __syncthreads();
    }
    if (wave != 0) return;
    // ---- first-reject scan and the record for the extra-token kernels (as accept_sequence)
    const int k = lane;
    const unsigned long long rej = __ballot(k < K && !acc);
    const bool any_nonfinite = __ballot(nonfinite) != 0ull;
    const bool any_bad = __ballot(bad) != 0ull;
    int n = rej ? (int)__builtin_ctzll(rej) : K;
    if (any_nonfinite) n = 0;
    if (k < K) out.out_tok[(int64_t)b * (K + 1) + k] = (k < n) ? tt : -1;
    if (k == 0) {
        out.out_tok[(int64_t)b * (K + 1) + K] = -1;
        out.n_accepted[b] = n;
        out.seq_status[b] = (any_nonfinite ? TLI_FLAG_NONFINITE : 0) | (any_bad ? TLI_FLAG_BAD_DRAFT : 0);
        out.fbad[b] = 0;
        if (out.lse_p) out.lse_p[(int64_t)b * (K + 1) + K] = NAN;
    }
    const bool residual = !any_nonfinite && n < K;
    if (residual ? (k == n) : (k == 0)) {
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
            f.l2p = my_lse * kLog2e;
            split_scale(in.c_t, f.rp.ct_hi, f.rp.ct_lo);
            split_hi_lo(f.l2p, f.rp.lp_hi, f.rp.lp_lo);
            if (!bad && (my_lq > -INFINITY || my_lq != my_lq)) {  // see accept_sequence
                f.rp.use_q = 1;
                split_scale(in.c_d, f.rp.cd_hi, f.rp.cd_lo);
                split_hi_lo(my_lq * kLog2e, f.rp.lq_hi, f.rp.lq_lo);
            }
        }
        out.frow[b] = f;
    }
}
