// tli_softmax_kernels.h -- Row normalisers, chunk tables and the inverse-CDF samplers: the drafting side of the path (q' of the
// intersection algorithm) and everything else that draws one token per softmax row.  Included by tli_kernels.hip
// inside its unnamed namespace, after tli_device_common.h.
#pragma once

// ---- kernel: log-normaliser partials of rows -----------------------------------------------------
// Standard SD appendix, verification loop: p_k(d_k) needs the normaliser of every target row k < K
// (MASKED = false).  With MASKED = true the same scan runs over drafter rows restricted to the shared
// ids (the normaliser of q' in the intersection algorithm), for callers that do not pass lse_q.
// grid (rows * nsplit); row r = (b, k) with b = r / K, k = r % K.
template <int DT, bool MASKED>
__global__ __launch_bounds__(kWG) void k_lse(const void* __restrict__ logits, int K, int64_t seq_stride,
                                              int64_t row_stride, int V, int nC, int cps, int nsplit, float cs,
                                              double ratio, const uint64_t* __restrict__ bits,
                                              Part* __restrict__ part, float2* __restrict__ ctab,
                                              int32_t* __restrict__ fbad = nullptr) {
    // (rows in memory order: position-major or reversed orders make no difference on rows that come from HBM)
    const int row = blockIdx.x / nsplit, split = blockIdx.x - row * nsplit;
    const int b = row / K, k = row - b * K;
    const u4v* rowv = reinterpret_cast<const u4v*>(static_cast<const char*>(logits) +
                                                    (b * seq_stride + k * row_stride) * Traits<DT>::ESZ);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const double kd = (ratio - 1.0) * kLn2;
    // verification without an accept kernel: the sequence's "drafter row of the residual holds NaN or +inf" flag
    // starts at 0 here (the residual scan's workgroups raise it, the draw reads it)
    if (fbad && k == 0 && split == 0 && threadIdx.x == 0) fbad[b] = 0;
    // The (ref, s) of every chunk is parked in LDS (no global store sits between the streaming loads, and the
    // running total is not advanced per chunk: that is a dozen fp64 instructions which every lane would
    // execute for a wave-uniform value); the partial is reduced from there when the row is through.  The pairs
    // are also what the residual of a rejected row takes its chunk sums of p from (ctab).
    extern __shared__ float2 stash[];  // min(cps, kLdsChunks) entries: a workgroup that keeps little LDS leaves the
                                       // CU's LDS to kernels running beside it
    Running over;  // chunks beyond what LDS parks (rows of more than kLdsChunks chunks per workgroup)
    scan_chunks<DT, MASKED, kWaves>(rowv, V, split * cps, min(nC, (split + 1) * cps), cs, (float)(ratio - 1.0), bits,
                                    [&](int c, float r, float sc) {
                                        const int i = c - split * cps;
                                        if (i < kLdsChunks) {
                                            if (lane == 0) stash[i] = make_float2(r, sc);
                                        } else {
                                            over.add(r, sc, kd);
                                            if (ctab && lane == 0) ctab[(int64_t)row * nC + c] = make_float2(r, sc);
                                        }
                                    });
    __shared__ float sref[kWaves];
    __shared__ double ssum[kWaves];
    __syncthreads();
    const int n_here = min(min(nC, (split + 1) * cps) - split * cps, kLdsChunks);
    float r_mine = over.ref;
    for (int i = threadIdx.x; i < n_here; i += kWG) {
        const float2 e = stash[i];
        r_mine = fmaxf(r_mine, e.x);
        if (ctab) ctab[(int64_t)row * nC + split * cps + i] = e;
    }
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
        part[(int64_t)row * nsplit + split] = p;
    }
}

// log-normaliser of a row from its partials: ln sum exp(x/temp) = ln2 * (ref * c_true/c + log2 S), where the
// factor c_true/c takes out the common part of the fp32 rounding of c.  NaN if a logit was NaN/+inf,
// -inf if the row has no mass.
// The partials are fetched kPartBatch at a time, all loads of a batch issued before the first is used (a loop of
// one load and its use per step is a chain of round trips: 32 of them for 16 partials); the arithmetic and its
// order are those of the plain loop.
constexpr int kPartBatch = 16;
__device__ __forceinline__ double combine_parts(const Part* pr, int nsplit, double ratio) {
    const double kd = (ratio - 1.0) * kLn2;
    Part first[kPartBatch];  // partials 0 .. kPartBatch - 1 (past the last: the last again), kept for both passes
#pragma unroll
    for (int u = 0; u < kPartBatch; ++u) first[u] = pr[min(u, nsplit - 1)];
    float R = first[0].ref;
#pragma unroll
    for (int u = 1; u < kPartBatch; ++u)
        if (u < nsplit) R = fmaxf(R, first[u].ref);
    for (int s0 = kPartBatch; s0 < nsplit; s0 += kPartBatch) {
        float r[kPartBatch];
#pragma unroll
        for (int u = 0; u < kPartBatch; ++u) r[u] = pr[min(s0 + u, nsplit - 1)].ref;
#pragma unroll
        for (int u = 0; u < kPartBatch; ++u)
            if (s0 + u < nsplit) R = fmaxf(R, r[u]);
    }
    double S = 0.0;
#pragma unroll
    for (int u = 0; u < kPartBatch; ++u)
        if (u < nsplit) S += first[u].s * exp2_diff(first[u].ref, R, kd);
    for (int s0 = kPartBatch; s0 < nsplit; s0 += kPartBatch) {
        Part q[kPartBatch];
#pragma unroll
        for (int u = 0; u < kPartBatch; ++u) q[u] = pr[min(s0 + u, nsplit - 1)];
#pragma unroll
        for (int u = 0; u < kPartBatch; ++u)
            if (s0 + u < nsplit) S += q[u].s * exp2_diff(q[u].ref, R, kd);
    }
    if (S != S || R == INFINITY) return NAN;
    if (!(S > 0.0)) return -INFINITY;
    return kLn2 * ((double)R * ratio + log2(S));
}

// kernel: lse[row] from the partials of k_lse.  grid (ceil(rows / 256)).
__global__ __launch_bounds__(kWG) void k_lse_finish(const Part* __restrict__ part, int rows, int nsplit, double ratio,
                                                     double* __restrict__ lse) {
    const int row = blockIdx.x * kWG + threadIdx.x;
    if (row < rows) lse[row] = combine_parts(part + (int64_t)row * nsplit, nsplit, ratio);
}

// ---- kernel: per-chunk (ref, s) table of a softmax row, optionally masked to the shared ids ----
// Used for drafter rows (masked: the intersection algorithm's q') and for the bonus target row.
// Workgroup `split` of a row owns chunks [split*cps, (split+1)*cps).
template <int DT, int MASKED>
__device__ __forceinline__ void table_scan(const u4v* rowv, int split, int V, int nC, int cps, float cs, double ratio,
                                           const uint64_t* bits,
                                  float* tab_ref, float* tab_s, float thr = -INFINITY) {
    const int lane = threadIdx.x & 63;
    scan_chunks<DT, MASKED, kWaves>(rowv, V, split * cps, min(nC, (split + 1) * cps), cs, (float)(ratio - 1.0), bits,
                                    [&](int c, float r, float sc) {
        if (lane == 0) { tab_ref[c] = r; tab_s[c] = sc; }
    }, thr);
}

template <int DT, int MASKED>
__global__ __launch_bounds__(kWG) void k_draft_scan(const void* __restrict__ logits, int64_t row_stride, int V,
                                                     int nC, int cps, int nsplit, float cs, double ratio,
                                                     const uint64_t* __restrict__ bits, float* __restrict__ tab_ref,
                                                     float* __restrict__ tab_s, const float* __restrict__ thr,
                                                     int64_t thr_stride) {
    const int row = blockIdx.x / nsplit, split = blockIdx.x - row * nsplit;
    const u4v* rowv = reinterpret_cast<const u4v*>(static_cast<const char*>(logits) +
                                                    (int64_t)row * row_stride * Traits<DT>::ESZ);
    table_scan<DT, MASKED>(rowv, split, V, nC, cps, cs, ratio, bits, tab_ref + (int64_t)row * nC,
                         tab_s + (int64_t)row * nC, (MASKED & 2) ? thr[(int64_t)row * thr_stride] : -INFINITY);
}

// ---- sampler: a workgroup of kLoads waves draws the token of a row from the row's chunk table ----
// (Every wave finds the chunk for itself -- a few hundred table entries, no barrier -- then the waves share
// the chosen chunk, one 16-byte load per lane each: the draw is a chain of dependent round trips to memory, and
// this takes three of them out of it.)

// exclusive prefix of v over the 64 lanes in fp64; *total = the wave's sum (uniform)
__device__ __forceinline__ double wave_excl_scan(double v, double* total) {
    const int lane = threadIdx.x & 63;
    double inc = v;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const double t = __shfl_up(inc, d, kWave);
        if (lane >= d) inc += t;
    }
    *total = __shfl(inc, kWave - 1, kWave);
    return inc - v;
}

__device__ __forceinline__ int wave_max_int(int v) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) v = max(v, __shfl_xor(v, d, kWave));
    return v;
}

// Chunk search.  Lane l owns the contiguous chunks [l*per, (l+1)*per); `mass(c)` is chunk c's fp64 mass.
// Returns the first chunk whose inclusive prefix exceeds theta = u * total, with theta - (prefix before
// it) in *theta_local; if rounding leaves no crossing, the last chunk with mass and +inf; -1 if the
// total is not positive (zero, negative or NaN).  All results are wave-uniform.
// P = chunks per lane held in registers: every mass is evaluated once, and a lane's loads (the chunk tables are in
// memory for some callers) are all issued before the first is used -- one round trip instead of one per chunk
// and pass.
template <int P, class MassFn>
__device__ __forceinline__ int find_chunk_p(int nC, int per, double u, MassFn mass, double* theta_local,
                                            double* total_out) {
    const int lane = threadIdx.x & 63;
    const int c0 = min(nC, lane * per), c1 = min(nC, c0 + per);
    double m[P];
    double mine = 0.0;
#pragma unroll
    for (int k = 0; k < P; ++k) {  // past the lane's range: some valid chunk is evaluated and dropped
        const double t = mass(min(c0 + k, nC - 1));
        m[k] = c0 + k < c1 ? t : 0.0;
    }
#pragma unroll
    for (int k = 0; k < P; ++k) mine += m[k];
    double total;
    const double excl = wave_excl_scan(mine, &total);
    *total_out = total;
    if (!(total > 0.0)) return -1;
    const double theta = u * total;
    double run = excl, before = 0.0;
    int found = -1, last_pos = -1;
#pragma unroll
    for (int k = 0; k < P; ++k) {
        const double t = m[k];
        if (t > 0.0) last_pos = c0 + k;
        if (found < 0 && c0 + k < c1 && run + t > theta) { found = c0 + k; before = run; }
        run += t;
    }
    const unsigned long long hit = __ballot(found >= 0);
    if (hit == 0ull) {
        *theta_local = INFINITY;
        return wave_max_int(last_pos);
    }
    const int src = (int)__builtin_ctzll(hit);  // lanes own ascending chunk ranges: lowest lane = first chunk
    *theta_local = theta - __shfl(before, src, kWave);
    return __shfl(found, src, kWave);
}

template <class MassFn>
__device__ __forceinline__ int find_chunk(int nC, double u, MassFn mass, double* theta_local, double* total_out) {
    const int lane = threadIdx.x & 63;
    const int per = (nC + kWave - 1) / kWave;
    if (per <= 2) return find_chunk_p<2>(nC, per, u, mass, theta_local, total_out);
    if (per <= 4) return find_chunk_p<4>(nC, per, u, mass, theta_local, total_out);
    const int c0 = min(nC, lane * per), c1 = min(nC, c0 + per);
    double mine = 0.0;
    for (int c = c0; c < c1; ++c) mine += mass(c);
    double total;
    const double excl = wave_excl_scan(mine, &total);
    *total_out = total;
    if (!(total > 0.0)) return -1;
    const double theta = u * total;
    double run = excl, before = 0.0;
    int found = -1, last_pos = -1;
    for (int c = c0; c < c1; ++c) {
        const double t = mass(c);
        if (t > 0.0) last_pos = c;
        if (found < 0 && run + t > theta) { found = c; before = run; }
        run += t;
    }
    const unsigned long long hit = __ballot(found >= 0);
    if (hit == 0ull) {
        *theta_local = INFINITY;
        return wave_max_int(last_pos);
    }
    const int src = (int)__builtin_ctzll(hit);  // lanes own ascending chunk ranges: lowest lane = first chunk
    *theta_local = theta - __shfl(before, src, kWave);
    return __shfl(found, src, kWave);
}

// In-chunk search by the kLoads waves of a workgroup.  The chunk's ids are taken in id order: load j = 0..3, then
// lane, then element; wave j holds load j, `w` = the weights of this lane's vector (ids e0 .. e0+N-1).  Returns
// (to every thread) the first id whose inclusive prefix exceeds theta_local, or, if rounding leaves no
// crossing, the last id with a positive weight (-1 if there is none).  The prefix over the loads is added up in
// load order, as one wave walking the four loads in turn would.  Every wave of the workgroup must call it; in a
// workgroup of more than kLoads waves the further ones take no part in the result (they only keep step at the
// barriers) and receive it like the others.
template <int N>
__device__ __forceinline__ int chunk_draw(const double (&w)[N], int64_t e0, double theta_local) {
    __shared__ double s_tot[kLoads];
    __shared__ int s_found[kLoads], s_last[kLoads];
    const int lane = threadIdx.x & 63;
    const int j = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    double mine = 0.0;
#pragma unroll
    for (int i = 0; i < N; ++i) mine += w[i];
    double tot;
    const double excl = wave_excl_scan(mine, &tot);
    if (lane == 0 && j < kLoads) s_tot[j] = tot;  // (a larger workgroup's further waves only keep step)
    __syncthreads();
    double base = 0.0;
    for (int q = 0; q < min(j, kLoads); ++q) base += s_tot[q];
    double run = base + excl;
    int f = -1, last_pos = -1;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        run += w[i];
        if (w[i] > 0.0) last_pos = (int)(e0 + i);
        if (f < 0 && run > theta_local) f = (int)(e0 + i);
    }
    const unsigned long long hit = __ballot(f >= 0);
    const int first = hit ? __shfl(f, (int)__builtin_ctzll(hit), kWave) : -1;
    const int last = wave_max_int(last_pos);
    if (lane == 0 && j < kLoads) { s_found[j] = first; s_last[j] = last; }
    __syncthreads();
    int tok = -1;
    for (int q = kLoads - 1; q >= 0; --q)
        if (s_found[q] >= 0) tok = s_found[q];  // the first load with a crossing
    if (tok < 0)
        for (int q = 0; q < kLoads; ++q) tok = max(tok, s_last[q]);
    return tok;
}

// weights of one 16-byte vector of a softmax row relative to reference `nref` (= -ref), as in
// reduce_chunk: 2^(x*c - ref); elements >= V or masked out get 0.
template <int DT, int MASKED>
__device__ __forceinline__ void softmax_vec_weights(const uint4* rowv, int64_t vi, int V, float cs, float nref,
                                                    const uint64_t* bits, double* w, float thr = -INFINITY) {
    constexpr int EPV = Traits<DT>::EPV;
    float x[EPV];
    if (vi * EPV < V) {
        unpack<DT>(rowv[vi], x);
        const uint32_t mb = (MASKED & 1) ? mask_bits<DT>(bits, vi) : 0xffu;  // same lane-mask words as the scan
#pragma unroll
        for (int i = 0; i < EPV; ++i) {
            const bool live = (vi * EPV + i < V) && ((mb >> i) & 1u) && !((MASKED & 2) && x[i] < thr);
            w[i] = live ? (double)exp2_hw(fmaf(x[i], cs, nref)) : 0.0;
        }
    } else {
#pragma unroll
        for (int i = 0; i < EPV; ++i) w[i] = 0.0;
    }
}

// Mass of a chunk of a softmax row relative to the row's reference M, from the chunk's table entry (ref, s).  A chunk
// whose reference lies more than kChunkFloor below M is given no mass: the draw forms the weights of a chunk's ids in
// fp32 relative to M, where those of such a chunk all flush to zero, and a draw that landed there -- u = 0 with such
// a chunk in front, u next to 1 with one at the end -- would find no id.  (All such chunks together hold less than
// 2^-100 of the row: the sum, and the normaliser formed from it, do not change.)  A chunk kept has an id of weight
// 2^-121 or more.  A NaN sum stays a NaN.
constexpr float kChunkFloor = 120.f;
__device__ __forceinline__ double chunk_mass(float ref, float s, float M, double kd) {
    if (ref < M - kChunkFloor && s == s) return 0.0;
    return (double)s * exp2_diff(ref, M, kd);
}

// Inverse-CDF sample of a (masked) softmax row from its chunk table, by the kLoads waves of a workgroup: every
// wave finds the chunk for itself (the table is small), then each takes one of the chunk's loads.  Returns the
// id, or -1 if the row has no usable mass (then *total_out is NaN for a NaN/+inf logit, else 0).  Every wave of
// the workgroup must call it, with the same arguments.
template <int DT, int MASKED>
__device__ __forceinline__ int sample_softmax_row(const void* rowp, int V, int nC, float cs, double ratio,
                                                  const uint64_t* bits,
                                                  const float* tr, const float* ts, double u, float* M_out,
                                                  double* total_out, float thr = -INFINITY) {
    constexpr int EPV = Traits<DT>::EPV;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float m = -INFINITY;
    for (int c = lane; c < nC; c += kWave) m = fmaxf(m, tr[c]);
    const float M = wave_max(m);
    *M_out = M;
    const double kd = (ratio - 1.0) * kLn2;
    double theta_local;
    const int c = find_chunk(nC, u, [&](int cc) { return chunk_mass(tr[cc], ts[cc], M, kd); }, &theta_local, total_out);
    if (c < 0) {
        if (M == INFINITY) *total_out = NAN;
        return -1;
    }
    const int64_t vi = ((int64_t)c * kLoads + wave) * kWave + lane;
    double w[EPV];
    if (wave < kLoads) {
        softmax_vec_weights<DT, MASKED>(static_cast<const uint4*>(rowp), vi, V, cs, -M, bits, w, thr);
    } else {
#pragma unroll
        for (int i = 0; i < EPV; ++i) w[i] = 0.0;
    }
    return chunk_draw<EPV>(w, vi * EPV, theta_local);
}

// ---- draft token of one drafter row from its chunk table ----------------------------------------
// Standard SD appendix, drafting loop, with q' of the intersection algorithm.
struct DraftOut {
    const float* u_draft;
    int32_t *tok_d, *tok_t;
    double *q_tok, *lse_q;
    int32_t* row_status;
    int64_t stride;  // entry of row r of every per-row array (u_draft and thr included) is at index r * stride
    const int32_t* r2d;  // compact rows: index in the row (= rank) -> drafter id; nullptr otherwise
    const float* thr;    // rows warped by threshold (MASKED bit 1): only logits >= thr[row] take part
};

// MASKED: the row is restricted to the shared ids (TLI's q').  Unmasked, the same code draws from the plain
// softmax of a row of any vocabulary: the union algorithm's draft (d2t then marks tokens outside T with -1)
// and the one-token-per-target-row draw of exact matching (d2t and tok_t null).
template <int DT, int MASKED>
__device__ __forceinline__ void draft_pick_row(const void* rowp, int row, int V, int nC, float cs, double c_ratio,
                                      double inv_temp, const uint64_t* bits, const int32_t* d2t, const float* tr,
                                      const float* ts, const DraftOut& o) {
    float M;
    double total;
    const int64_t at = (int64_t)row * o.stride;
    const int d = sample_softmax_row<DT, MASKED>(rowp, V, nC, cs, c_ratio, bits, tr, ts, (double)o.u_draft[at], &M, &total,
                                                 (MASKED & 2) ? o.thr[at] : -INFINITY);
    if (threadIdx.x != 0) return;
    if (d < 0) {  // no usable mass: NaN/+inf among the logits that take part, or all of them -inf
        const bool nonfinite = (total != total);
        o.tok_d[at] = -1;
        if (o.tok_t) o.tok_t[at] = -1;
        if (o.q_tok) o.q_tok[at] = 0.0;
        if (o.lse_q) o.lse_q[at] = nonfinite ? NAN : -INFINITY;
        o.row_status[at] = nonfinite ? TLI_FLAG_NONFINITE : TLI_FLAG_ZERO_MASS;
        return;
    }
    const double lse = kLn2 * ((double)M * c_ratio + log2(total));
    const int id = o.r2d ? o.r2d[d] : d;  // the id reported: a drafter id also when the row is in compact layout
    o.tok_d[at] = id;
    if (o.tok_t) o.tok_t[at] = d2t ? d2t[id] : id;
    if (o.lse_q) o.lse_q[at] = lse;
    if (o.q_tok) o.q_tok[at] = exp((double)load_elem<DT>(rowp, d) * inv_temp - lse);
    o.row_status[at] = 0;
}

// kernel: sampler of the split path (rows cut over several workgroups by k_draft_scan).  grid (R), kLoads waves.
template <int DT, int MASKED>
__global__ __launch_bounds__(kLoads * kWave) void k_draft_pick(const void* __restrict__ logits, int64_t row_stride, int V,
                                                     int nC, float cs, double c_ratio, double inv_temp,
                                                     const uint64_t* __restrict__ bits,
                                                     const int32_t* __restrict__ d2t,
                                                     const float* __restrict__ tab_ref,
                                                     const float* __restrict__ tab_s, DraftOut o) {
    const int row = blockIdx.x;
    const char* rowp = static_cast<const char*>(logits) + (int64_t)row * row_stride * Traits<DT>::ESZ;
    draft_pick_row<DT, MASKED>(rowp, row, V, nC, cs, c_ratio, inv_temp, bits, d2t, tab_ref + (int64_t)row * nC,
                       tab_s + (int64_t)row * nC, o);
}

// kernel: one workgroup per drafter row scans it into a chunk table in LDS and samples from it at
// once, while the other workgroups on the CU keep streaming their rows.
// grid (R); nC <= kLdsChunks.
template <int DT, int MASKED>
__global__ __launch_bounds__(kWG) void k_draft_fused(const void* __restrict__ logits, int64_t row_stride, int V,
                                                      int nC, float cs, double c_ratio, double inv_temp,
                                                      const uint64_t* __restrict__ bits,
                                                      const int32_t* __restrict__ d2t, DraftOut o) {
    __shared__ float tr[kLdsChunks], ts[kLdsChunks];
    const int row = blockIdx.x;
    const char* rowp = static_cast<const char*>(logits) + (int64_t)row * row_stride * Traits<DT>::ESZ;
    table_scan<DT, MASKED>(reinterpret_cast<const u4v*>(rowp), 0, V, nC, nC, cs, c_ratio, bits, tr, ts,
                           (MASKED & 2) ? o.thr[(int64_t)row * o.stride] : -INFINITY);
    __syncthreads();
    draft_pick_row<DT, MASKED>(rowp, row, V, nC, cs, c_ratio, inv_temp, bits, d2t, tr, ts, o);
}

// ---- few short rows: a row per workgroup of sixteen waves, held in registers -----------------------
// Standard SD appendix, drafting loop, for calls of few rows of a small vocabulary (a single sequence's lookahead,
// or one position of a batch): the rows do not fill the chip, and what counts is the call's latency -- one kernel
// instead of two.  Wave w of the row's workgroup loads the chunks w and w + 16 in one go and keeps them: the chunk
// table goes to LDS, every wave finds the chunk of the draw, and the wave that holds it draws from its registers --
// no second trip to memory for the chunk, its mask words or the drawn logit.  The arithmetic, and its order, are
// those of the split kernels (reduce_chunk, find_chunk, chunk_draw with one wave standing in for the four in turn),
// so the results are the same to the bit.  Measured per call, R rows of 32,000 fp32 logits: 10.7 us against 13.7 us
// for scan + draw in two kernels, for every R from 1 to 256 (512 rows: 19.6 against 15.8 us).  With four chunks per
// wave (rows of 128,256 bf16 logits) the two kernels win from 5 rows on, so such rows keep them.
// Rows of up to kRowChunks chunks; grid (R).
constexpr int kRowWaves = 16;
constexpr int kRowSets = 2;
constexpr int kRowChunks = kRowWaves * kRowSets;
constexpr int kRowMaxRows = 256;

// chunk_draw by one wave that holds all kLoads vectors of the chunk (x[j * N + i]: element i of load j, id
// c0_elem + (j * 64 + lane) * N + i; -inf for ids that take no part).  *x_out: the logit of the id returned, set in
// the lane that holds it (*mine_out).
template <int N>
__device__ __forceinline__ int chunk_draw_wave(const float (&x)[kLoads * N], float cs, float nref, int64_t c0_elem,
                                               double theta_local, float* x_out, bool* mine_out) {
    const int lane = threadIdx.x & 63;
    double base = 0.0;
    int tok = -1, last = -1;
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        double w[N];
        double mine = 0.0;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            w[i] = (double)exp2_hw(fmaf(x[j * N + i], cs, nref));  // (-inf, an id that takes no part: 0)
            mine += w[i];
        }
        double tot;
        const double excl = wave_excl_scan(mine, &tot);
        const int64_t e0 = c0_elem + ((int64_t)j * kWave + lane) * N;
        double run = base + excl;
        int f = -1, last_pos = -1;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            run += w[i];
            if (w[i] > 0.0) last_pos = (int)(e0 + i);
            if (f < 0 && run > theta_local) f = (int)(e0 + i);
        }
        const unsigned long long hit = __ballot(f >= 0);
        const int first = hit ? __shfl(f, (int)__builtin_ctzll(hit), kWave) : -1;
        if (tok < 0 && first >= 0) tok = first;  // the first load with a crossing
        last = max(last, wave_max_int(last_pos));
        base += tot;
    }
    if (tok < 0) tok = last;
    *mine_out = false;
    if (tok >= 0) {
        const int64_t rel = tok - c0_elem;  // (j * 64 + lane) * N + i
        const int jj = (int)(rel / (kWave * N)), ll = (int)((rel / N) % kWave), ii = (int)(rel % N);
        if (ll == lane) {
            float v = 0.f;
#pragma unroll
            for (int q = 0; q < kLoads * N; ++q)
                if (q == jj * N + ii) v = x[q];
            *x_out = v;
            *mine_out = true;
        }
    }
    return tok;
}

template <int DT, int MASKED>
__global__ __launch_bounds__(kRowWaves * kWave) void k_draft_row(const void* __restrict__ logits, int64_t row_stride, int V,
                                                                int nC, float cs, double c_ratio, double inv_temp,
                                                                const uint64_t* __restrict__ bits,
                                                                const int32_t* __restrict__ d2t, DraftOut o) {
    constexpr int EPV = Traits<DT>::EPV;
    constexpr int N = EPV * kLoads;
    __shared__ float tr[kRowChunks], ts[kRowChunks];
    __shared__ int s_tok;
    __shared__ float s_x;
    const int row = blockIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int64_t at = (int64_t)row * o.stride;
    const u4v* rowv = reinterpret_cast<const u4v*>(static_cast<const char*>(logits) + (int64_t)row * row_stride * Traits<DT>::ESZ);
    const float thr = (MASKED & 2) ? o.thr[at] : -INFINITY;
    const float dl = (float)(c_ratio - 1.0);
    const int n_whole = V / chunk_elems<DT>();
    const int nvec = (V + EPV - 1) / EPV;
    ChunkRegs regs[kRowSets];
#pragma unroll
    for (int q = 0; q < kRowSets; ++q) {  // every load of the wave is issued before the first is used
        const int c = wave + q * kRowWaves;
        if (c < n_whole) load_chunk_whole(rowv, c, lane, regs[q]);
        else if (c < nC) load_chunk_tail<DT>(rowv, c, lane, nvec, regs[q]);
    }
#pragma unroll
    for (int q = 0; q < kRowSets; ++q) {
        const int c = wave + q * kRowWaves;
        if (c < nC) {
            float ref, sum;
            if (c < n_whole) reduce_chunk<DT, MASKED, true>(regs[q], c, lane, V, cs, dl, bits, ref, sum, thr);
            else reduce_chunk<DT, MASKED, false>(regs[q], c, lane, V, cs, dl, bits, ref, sum, thr);
            if (lane == 0) { tr[c] = ref; ts[c] = sum; }
        }
    }
    if (threadIdx.x == 0) s_tok = -1;
    __syncthreads();
    // every wave: the chunk of the draw (as sample_softmax_row)
    float m = -INFINITY;
    for (int c = lane; c < nC; c += kWave) m = fmaxf(m, tr[c]);
    const float M = wave_max(m);
    const double kd = (c_ratio - 1.0) * kLn2;
    double theta_local, total;
    const int cs_chunk = find_chunk(nC, (double)o.u_draft[at], [&](int cc) { return chunk_mass(tr[cc], ts[cc], M, kd); },
                                    &theta_local, &total);
    if (cs_chunk >= 0 && wave == cs_chunk % kRowWaves) {  // the wave that holds it
        const int q_sel = cs_chunk / kRowWaves;
        float x[N];
#pragma unroll
        for (int q = 0; q < kRowSets; ++q)
            if (q == q_sel) {  // (wave-uniform: the register set is picked by a branch, not by an index)
                if (cs_chunk < n_whole) chunk_values<DT, (MASKED & 1) != 0, true>(regs[q], cs_chunk, lane, V, bits, x);
                else chunk_values<DT, (MASKED & 1) != 0, false>(regs[q], cs_chunk, lane, V, bits, x);
            }
        if (MASKED & 2) {
#pragma unroll
            for (int i = 0; i < N; ++i) x[i] = x[i] < thr ? -INFINITY : x[i];
        }
        float xv = 0.f;
        bool mine;
        const int tok = chunk_draw_wave<EPV>(x, cs, -M, (int64_t)cs_chunk * chunk_elems<DT>(), theta_local, &xv, &mine);
        if (mine) { s_x = xv; s_tok = tok; }
    }
    __syncthreads();
    if (threadIdx.x != 0) return;
    const int d = s_tok;
    if (cs_chunk < 0 || d < 0) {  // no usable mass: NaN/+inf among the logits that take part, or all of them -inf
        const bool nonfinite = (total != total) || M == INFINITY;
        o.tok_d[at] = -1;
        if (o.tok_t) o.tok_t[at] = -1;
        if (o.q_tok) o.q_tok[at] = 0.0;
        if (o.lse_q) o.lse_q[at] = nonfinite ? NAN : -INFINITY;
        o.row_status[at] = nonfinite ? TLI_FLAG_NONFINITE : TLI_FLAG_ZERO_MASS;
        return;
    }
    const double lse = kLn2 * ((double)M * c_ratio + log2(total));
    const int id = o.r2d ? o.r2d[d] : d;
    o.tok_d[at] = id;
    if (o.tok_t) o.tok_t[at] = d2t ? d2t[id] : id;
    if (o.lse_q) o.lse_q[at] = lse;
    if (o.q_tok) o.q_tok[at] = exp((double)s_x * inv_temp - lse);
    o.row_status[at] = 0;
}
