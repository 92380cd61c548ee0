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
#include <new>
#include <type_traits>
#include <vector>

#include "tli.h"

namespace {

constexpr int kWave = 64;
constexpr int kWG = 256;
constexpr int kWaves = kWG / kWave;
constexpr int kLoads = 4;
constexpr int kMaxK = 64;
constexpr int kLdsChunks = 1024;  // chunk-table entries a workgroup may park in LDS
constexpr double kLn2 = 0.693147180559945309417232121458;
constexpr double kLog2e = 1.44269504088896340735992468100;

template <int DT> struct Traits;
template <> struct Traits<TLI_F32> {
    static constexpr int EPV = 4;  // elements per 16-byte vector
    static constexpr int ESZ = 4;
};
template <> struct Traits<TLI_BF16> {
    static constexpr int EPV = 8;
    static constexpr int ESZ = 2;
};
template <int DT> constexpr int chunk_elems() { return kWave * kLoads * Traits<DT>::EPV; }

__device__ __forceinline__ float as_f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u(float f) { return __builtin_bit_cast(uint32_t, f); }

template <int DT> __device__ __forceinline__ void unpack(const uint4& v, float* x);
template <> __device__ __forceinline__ void unpack<TLI_F32>(const uint4& v, float* x) {
    x[0] = as_f(v.x); x[1] = as_f(v.y); x[2] = as_f(v.z); x[3] = as_f(v.w);
}
template <> __device__ __forceinline__ void unpack<TLI_BF16>(const uint4& v, float* x) {
    x[0] = as_f(v.x << 16); x[1] = as_f(v.x & 0xffff0000u);
    x[2] = as_f(v.y << 16); x[3] = as_f(v.y & 0xffff0000u);
    x[4] = as_f(v.z << 16); x[5] = as_f(v.z & 0xffff0000u);
    x[6] = as_f(v.w << 16); x[7] = as_f(v.w & 0xffff0000u);
}

template <int DT> __device__ __forceinline__ float load_elem(const void* base, int64_t idx);
template <> __device__ __forceinline__ float load_elem<TLI_F32>(const void* base, int64_t idx) {
    return static_cast<const float*>(base)[idx];
}
template <> __device__ __forceinline__ float load_elem<TLI_BF16>(const void* base, int64_t idx) {
    return as_f(static_cast<uint32_t>(static_cast<const uint16_t*>(base)[idx]) << 16);
}

// ---- wave64 reductions on the DPP network (result broadcast through an SGPR) -------------------
template <int CTRL, int ROW_MASK> __device__ __forceinline__ float dpp(float old, float v) {
    return as_f(__builtin_amdgcn_update_dpp(as_u(old), as_u(v), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp<0xB1, 0xF>(0.f, v);   // quad_perm [1,0,3,2]
    v += dpp<0x4E, 0xF>(0.f, v);   // quad_perm [2,3,0,1]
    v += dpp<0x124, 0xF>(0.f, v);  // row_ror 4
    v += dpp<0x128, 0xF>(0.f, v);  // row_ror 8
    v += dpp<0x142, 0xA>(0.f, v);  // row_bcast 15 into rows 1,3
    v += dpp<0x143, 0xC>(0.f, v);  // row_bcast 31 into rows 2,3
    return as_f(__builtin_amdgcn_readlane(as_u(v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
    const float ninf = -INFINITY;
    v = fmaxf(v, dpp<0xB1, 0xF>(ninf, v));
    v = fmaxf(v, dpp<0x4E, 0xF>(ninf, v));
    v = fmaxf(v, dpp<0x124, 0xF>(ninf, v));
    v = fmaxf(v, dpp<0x128, 0xF>(ninf, v));
    v = fmaxf(v, dpp<0x142, 0xA>(ninf, v));
    v = fmaxf(v, dpp<0x143, 0xC>(ninf, v));
    return as_f(__builtin_amdgcn_readlane(as_u(v), 63));
}

// the same network for a double: its two halves travel separately (DPP moves 32-bit registers)
template <int CTRL, int ROW_MASK> __device__ __forceinline__ double dpp_f64(double v) {
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = __builtin_amdgcn_update_dpp(0u, (uint32_t)b, CTRL, ROW_MASK, 0xF, false);
    const uint32_t hi = __builtin_amdgcn_update_dpp(0u, (uint32_t)(b >> 32), CTRL, ROW_MASK, 0xF, false);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);  // lanes outside ROW_MASK receive +0.0
}
__device__ __forceinline__ double wave_sum_f64(double v) {
    v += dpp_f64<0xB1, 0xF>(v);
    v += dpp_f64<0x4E, 0xF>(v);
    v += dpp_f64<0x124, 0xF>(v);
    v += dpp_f64<0x128, 0xF>(v);
    v += dpp_f64<0x142, 0xA>(v);
    v += dpp_f64<0x143, 0xC>(v);
    const uint64_t b = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)b, 63), hi = __builtin_amdgcn_readlane((uint32_t)(b >> 32), 63);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ float exp2_hw(float x) { return __builtin_amdgcn_exp2f(x); }

// ---- chunk loads ------------------------------------------------------------------------------
// Chunk c of a row = vectors [c*256, c*256+256); load j of lane l is vector c*256 + j*64 + l.
// Rows are streamed once, so the loads are non-temporal (they bypass cache allocation).
typedef unsigned int u4v __attribute__((ext_vector_type(4)));

struct ChunkRegs {
    u4v v[kLoads];
};

__device__ __forceinline__ uint4 to_uint4(const u4v& t) { return make_uint4(t.x, t.y, t.z, t.w); }

// whole chunk: every vector is in range, no guards
__device__ __forceinline__ void load_chunk_whole(const u4v* rowv, int c, int lane, ChunkRegs& r) {
    const u4v* p = rowv + (int64_t)c * (kWave * kLoads) + lane;
#pragma unroll
    for (int j = 0; j < kLoads; ++j) r.v[j] = __builtin_nontemporal_load(p + j * kWave);
}

// last, partial chunk of a row: vectors past the end read as -inf
template <int DT>
__device__ __forceinline__ void load_chunk_tail(const u4v* rowv, int c, int lane, int nvec, ChunkRegs& r) {
    const unsigned int pat = (DT == TLI_BF16) ? 0xff80ff80u : 0xff800000u;
    const int64_t v0 = (int64_t)c * (kWave * kLoads) + lane;
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        const int64_t vi = v0 + j * kWave;
        u4v t = {pat, pat, pat, pat};
        if (vi < nvec) t = rowv[vi];
        r.v[j] = t;
    }
}

// Shared-id mask in "lane mask" layout: for chunk c, load j and element i of a vector, the 64-bit word
// lmask[(c*kLoads + j)*EPV + i] has bit l set iff the id held by lane l there -- id
// ((c*kLoads + j)*64 + l)*EPV + i -- is shared (ids past the vocabulary read as not shared).  A wave
// fetches the word with one scalar load and uses it directly as the select mask of a v_cndmask.
template <int DT> __device__ __forceinline__ uint32_t mask_bits(const uint64_t* lmask, int64_t vi) {
    constexpr int EPV = Traits<DT>::EPV;
    const uint64_t* w = lmask + (vi >> 6) * EPV;
    const int l = (int)(vi & 63);
    uint32_t mb = 0;
#pragma unroll
    for (int i = 0; i < EPV; ++i) mb |= (uint32_t)((w[i] >> l) & 1ull) << i;
    return mb;
}

// Reduce one chunk held in registers to (ref, s): sum 2^(x*c) over the chunk = s * 2^ref, with
// ref = ceil(max over the chunk of fp32(x*c)) (-inf and s = 0 for a chunk without finite entries).
// A NaN or +inf logit turns s into NaN.  Wave-uniform results.  WHOLE: every element is < V.
template <int DT, bool MASKED, bool WHOLE>
__device__ __forceinline__ void reduce_chunk(const ChunkRegs& r, int c, int lane, int V, float cs, float dl,
                                             const uint64_t* bits, float& ref_out, float& s_out) {
    constexpr int EPV = Traits<DT>::EPV;
    constexpr int N = EPV * kLoads;
    float x[N];
    const int64_t v0 = (int64_t)c * (kWave * kLoads) + lane;
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        unpack<DT>(to_uint4(r.v[j]), x + j * EPV);
        const int64_t vi = v0 + j * kWave;
        if (!WHOLE) {
#pragma unroll
            for (int i = 0; i < EPV; ++i)
                if (vi * EPV + i >= V) x[j * EPV + i] = -INFINITY;
        }
        if (MASKED) {
            const uint64_t* w = bits + ((int64_t)c * kLoads + j) * EPV;  // wave-uniform address: scalar loads
#pragma unroll
            for (int i = 0; i < EPV; ++i) {
                const bool keep = __builtin_amdgcn_inverse_ballot_w64(w[i]);
                x[j * EPV + i] = keep ? x[j * EPV + i] : -INFINITY;
            }
        }
    }
    float m = x[0];
#pragma unroll
    for (int i = 1; i < N; ++i) m = fmaxf(m, x[i]);
    // ref must be THE rounded product that the fma below subtracts.  (Built with -ffp-contract=off: fused into
    // the later `ref - R`, the multiply would enter there unrounded and the lane's sum would be rescaled
    // against a reference it was not formed with -- an error of up to 1.4e-6, measured.)
    const float ref = m * cs;
    const float nref = (m == -INFINITY) ? 0.f : -ref;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i & 3] += exp2_hw(fmaf(x[i], cs, nref));
    float s = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    // the chunk's reference is rounded up to an integer: every later rescaling between references is then
    // an exact power of two (ldexp), in fp32 and fp64 alike
    const float R = ceilf(wave_max(ref));
    // (1 + dl) = c_true / c: the lane is moved to the chunk reference in the TRUE scale, which takes the
    // fp32 rounding of c out of everything but the spread of logits inside one lane
    const float e = ref - R;
    s = (m == -INFINITY) ? 0.f : s * exp2_hw(fmaf(e, dl, e));
    ref_out = R;
    s_out = wave_sum(s);
}

// Stream the chunks c_begin + wave, + NW, ... < c_end of one row (NW = waves in the workgroup) through
// `proc(regs, c, whole)` (whole: std::true_type if every element of the chunk is < V).  Whole chunks run in
// a two-stage register pipeline: the loads of the next chunk are in flight while the current one is
// processed.  A row has at most one partial chunk (its last); the wave that owns it handles it after its
// whole chunks.
template <int DT, int NW, class Proc>
__device__ __forceinline__ void stream_chunks(const u4v* rowv, int V, int c_begin, int c_end, Proc&& proc) {
    constexpr int EPV = Traits<DT>::EPV;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int n_whole = V / chunk_elems<DT>();
    const int hot_end = min(c_end, n_whole);
    int c = c_begin + wave;
    if (c < hot_end) {
        ChunkRegs a, b;
        load_chunk_whole(rowv, c, lane, a);
        while (true) {
            if (c + NW >= hot_end) {
                proc(a, c, std::true_type());
                c += NW;
                break;
            }
            load_chunk_whole(rowv, c + NW, lane, b);
            proc(a, c, std::true_type());
            c += NW;
            if (c + NW >= hot_end) {
                proc(b, c, std::true_type());
                c += NW;
                break;
            }
            load_chunk_whole(rowv, c + NW, lane, a);
            proc(b, c, std::true_type());
            c += NW;
        }
    }
    if (c < c_end) {  // c == n_whole: the partial chunk
        ChunkRegs t;
        load_chunk_tail<DT>(rowv, c, lane, (V + EPV - 1) / EPV, t);
        proc(t, c, std::false_type());
    }
}

// the softmax scan: every chunk reduced to (ref, s) and handed to `sink(c, ref, s)`
template <int DT, bool MASKED, int NW, class Sink>
__device__ __forceinline__ void scan_chunks(const u4v* rowv, int V, int c_begin, int c_end, float cs, float dl,
                                            const uint64_t* bits, Sink&& sink) {
    const int lane = threadIdx.x & 63;
    stream_chunks<DT, NW>(rowv, V, c_begin, c_end, [&](const ChunkRegs& r, int c, auto whole) {
        float ref, sum;
        reduce_chunk<DT, MASKED, decltype(whole)::value>(r, c, lane, V, cs, dl, bits, ref, sum);
        sink(c, ref, sum);
    });
}

// 2^((a-b) * c_true/c) for integer-valued references a <= b (or -inf / +inf), with c_true/c = 1 + delta and
// kd = delta * ln 2: an exact ldexp times the first-order factor (delta ~ 1e-8, the rest is < 1e-12).
// 0 if a = -inf, NaN if both are +inf.
__device__ __forceinline__ double exp2_diff(float a, float b, double kd) {
    if (a == -INFINITY) return 0.0;
    const float d = a - b;
    if (d != d) return NAN;
    const float dc = fmaxf(d, -1100.f);
    return ldexp(1.0 + kd * (double)dc, (int)dc);
}

// running (ref, sum) of a wave, sum kept in fp64
struct Running {
    float ref = -INFINITY;
    double s = 0.0;
    __device__ __forceinline__ void add(float r, float sc, double kd) {
        const float nr = fmaxf(ref, r);
        if (nr == -INFINITY) return;
        s = s * exp2_diff(ref, nr, kd) + (double)sc * exp2_diff(r, nr, kd);
        ref = nr;
    }
};

struct Part {  // partial log-normaliser of (a split of) a row: sum 2^(x*c) = s * 2^ref
    float ref;
    float pad;
    double s;
};


// ---- kernel: log-normaliser partials of rows -----------------------------------------------------
// Standard SD appendix, verification loop: p_k(d_k) needs the normaliser of every target row k < K
// (MASKED = false).  With MASKED = true the same scan runs over drafter rows restricted to the shared
// ids (the normaliser of q' in the intersection algorithm), for callers that do not pass lse_q.
// grid (rows * nsplit); row r = (b, k) with b = r / K, k = r % K.
template <int DT, bool MASKED>
__global__ __launch_bounds__(kWG) void k_lse(const void* __restrict__ logits, int K, int64_t seq_stride,
                                              int64_t row_stride, int V, int nC, int cps, int nsplit, float cs,
                                              double ratio, const uint64_t* __restrict__ bits,
                                              Part* __restrict__ part, float2* __restrict__ ctab) {
    const int row = blockIdx.x / nsplit, split = blockIdx.x - row * nsplit;
    const int b = row / K, k = row - b * K;
    const u4v* rowv = reinterpret_cast<const u4v*>(static_cast<const char*>(logits) +
                                                    (b * seq_stride + k * row_stride) * Traits<DT>::ESZ);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const double kd = (ratio - 1.0) * kLn2;
    // The (ref, s) of every chunk is parked in LDS (no global store sits between the streaming loads, and the
    // running total is not advanced per chunk: that is a dozen fp64 instructions which every lane would
    // execute for a wave-uniform value); the partial is reduced from there when the row is through.  The pairs
    // are also what the residual of a rejected row takes its chunk sums of p from (ctab).
    __shared__ float2 stash[kLdsChunks];
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
__device__ __forceinline__ double combine_parts(const Part* pr, int nsplit, double ratio) {
    float R = pr[0].ref;
    for (int s = 1; s < nsplit; ++s) R = fmaxf(R, pr[s].ref);
    double S = 0.0;
    for (int s = 0; s < nsplit; ++s) S += pr[s].s * exp2_diff(pr[s].ref, R, (ratio - 1.0) * kLn2);
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
template <int DT, bool MASKED>
__device__ __forceinline__ void table_scan(const u4v* rowv, int split, int V, int nC, int cps, float cs, double ratio,
                                           const uint64_t* bits,
                                  float* tab_ref, float* tab_s) {
    const int lane = threadIdx.x & 63;
    scan_chunks<DT, MASKED, kWaves>(rowv, V, split * cps, min(nC, (split + 1) * cps), cs, (float)(ratio - 1.0), bits,
                                    [&](int c, float r, float sc) {
        if (lane == 0) { tab_ref[c] = r; tab_s[c] = sc; }
    });
}

template <int DT, bool MASKED>
__global__ __launch_bounds__(kWG) void k_draft_scan(const void* __restrict__ logits, int64_t row_stride, int V,
                                                     int nC, int cps, int nsplit, float cs, double ratio,
                                                     const uint64_t* __restrict__ bits, float* __restrict__ tab_ref,
                                                     float* __restrict__ tab_s) {
    const int row = blockIdx.x / nsplit, split = blockIdx.x - row * nsplit;
    const u4v* rowv = reinterpret_cast<const u4v*>(static_cast<const char*>(logits) +
                                                    (int64_t)row * row_stride * Traits<DT>::ESZ);
    table_scan<DT, MASKED>(rowv, split, V, nC, cps, cs, ratio, bits, tab_ref + (int64_t)row * nC,
                         tab_s + (int64_t)row * nC);
}

// ---- wave-level sampler: one wave draws the token of a row from the row's chunk table ----------
// (One wave is enough for a few hundred chunks and one 2048-id chunk; it needs no barriers, and in
// the fused draft kernel the other three waves of the workgroup retire at once.)

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
// load order, as one wave walking the four loads in turn would.  Every wave of the workgroup must call it.
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
    if (lane == 0) s_tot[j] = tot;
    __syncthreads();
    double base = 0.0;
    for (int q = 0; q < j; ++q) base += s_tot[q];
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
    if (lane == 0) { s_found[j] = first; s_last[j] = last; }
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
template <int DT, bool MASKED>
__device__ __forceinline__ void softmax_vec_weights(const uint4* rowv, int64_t vi, int V, float cs, float nref,
                                                    const uint64_t* bits, double* w) {
    constexpr int EPV = Traits<DT>::EPV;
    float x[EPV];
    if (vi * EPV < V) {
        unpack<DT>(rowv[vi], x);
        const uint32_t mb = MASKED ? mask_bits<DT>(bits, vi) : 0xffu;  // same lane-mask words as the scan
#pragma unroll
        for (int i = 0; i < EPV; ++i) {
            const bool live = (vi * EPV + i < V) && ((mb >> i) & 1u);
            w[i] = live ? (double)exp2_hw(fmaf(x[i], cs, nref)) : 0.0;
        }
    } else {
#pragma unroll
        for (int i = 0; i < EPV; ++i) w[i] = 0.0;
    }
}

// Inverse-CDF sample of a (masked) softmax row from its chunk table, by the kLoads waves of a workgroup: every
// wave finds the chunk for itself (the table is small), then each takes one of the chunk's loads.  Returns the
// id, or -1 if the row has no usable mass (then *total_out is NaN for a NaN/+inf logit, else 0).  Every wave of
// the workgroup must call it, with the same arguments.
template <int DT, bool MASKED>
__device__ __forceinline__ int sample_softmax_row(const void* rowp, int V, int nC, float cs, double ratio,
                                                  const uint64_t* bits,
                                                  const float* tr, const float* ts, double u, float* M_out,
                                                  double* total_out) {
    constexpr int EPV = Traits<DT>::EPV;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float m = -INFINITY;
    for (int c = lane; c < nC; c += kWave) m = fmaxf(m, tr[c]);
    const float M = wave_max(m);
    *M_out = M;
    const double kd = (ratio - 1.0) * kLn2;
    double theta_local;
    const int c = find_chunk(nC, u, [&](int cc) { return (double)ts[cc] * exp2_diff(tr[cc], M, kd); }, &theta_local,
                             total_out);
    if (c < 0) {
        if (M == INFINITY) *total_out = NAN;
        return -1;
    }
    const int64_t vi = ((int64_t)c * kLoads + wave) * kWave + lane;
    double w[EPV];
    softmax_vec_weights<DT, MASKED>(static_cast<const uint4*>(rowp), vi, V, cs, -M, bits, w);
    return chunk_draw<EPV>(w, vi * EPV, theta_local);
}

// ---- draft token of one drafter row from its chunk table ----------------------------------------
// Standard SD appendix, drafting loop, with q' of the intersection algorithm.
struct DraftOut {
    const float* u_draft;
    int32_t *tok_d, *tok_t;
    double *q_tok, *lse_q;
    int32_t* row_status;
    int64_t stride;  // entry of row r of every per-row array (u_draft included) is at index r * stride
    const int32_t* r2d;  // compact rows: index in the row (= rank) -> drafter id; nullptr otherwise
};

// MASKED: the row is restricted to the shared ids (TLI's q').  Unmasked, the same code draws from the plain
// softmax of a row of any vocabulary: the union algorithm's draft (d2t then marks tokens outside T with -1)
// and the one-token-per-target-row draw of exact matching (d2t and tok_t null).
template <int DT, bool MASKED>
__device__ __forceinline__ void draft_pick_row(const void* rowp, int row, int V, int nC, float cs, double c_ratio,
                                      double inv_temp, const uint64_t* bits, const int32_t* d2t, const float* tr,
                                      const float* ts, const DraftOut& o) {
    float M;
    double total;
    const int64_t at = (int64_t)row * o.stride;
    const int d = sample_softmax_row<DT, MASKED>(rowp, V, nC, cs, c_ratio, bits, tr, ts, (double)o.u_draft[at], &M, &total);
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
template <int DT, bool MASKED>
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
template <int DT, bool MASKED>
__global__ __launch_bounds__(kWG) void k_draft_fused(const void* __restrict__ logits, int64_t row_stride, int V,
                                                      int nC, float cs, double c_ratio, double inv_temp,
                                                      const uint64_t* __restrict__ bits,
                                                      const int32_t* __restrict__ d2t, DraftOut o) {
    __shared__ float tr[kLdsChunks], ts[kLdsChunks];
    const int row = blockIdx.x;
    const char* rowp = static_cast<const char*>(logits) + (int64_t)row * row_stride * Traits<DT>::ESZ;
    table_scan<DT, MASKED>(reinterpret_cast<const u4v*>(rowp), 0, V, nC, nC, cs, c_ratio, bits, tr, ts);
    __syncthreads();
    draft_pick_row<DT, MASKED>(rowp, row, V, nC, cs, c_ratio, inv_temp, bits, d2t, tr, ts, o);
}

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

// ---- kernel: accept tests and first-reject scan ------------------------------------------------
// Standard SD appendix, verification loop and the count of accepted drafts.  grid (B), 64 threads;
// lane k owns position k.
template <int DT>
__global__ __launch_bounds__(kWave) void k_accept(const void* __restrict__ logits_t, DrafterView dv,
                                                   int K, int Vt, int Vd, int nsplit, const Part* __restrict__ part,
                                                   double ratio_t, double inv_temp_t, double inv_temp_d,
                                                   const int32_t* __restrict__ d2t, const int32_t* __restrict__ tok_d,
                                                   const double* __restrict__ lse_q, const float* __restrict__ u_acc,
                                                   int32_t* __restrict__ n_accepted, int32_t* __restrict__ out_tok,
                                                   uint8_t* __restrict__ accept, double* __restrict__ p_tok,
                                                   double* __restrict__ q_tok, double* __restrict__ lse_p,
                                                   int32_t* __restrict__ seq_status, double* __restrict__ ws_lse_p, double c_t,
                                                   double c_d, FinalRow* __restrict__ frow, int32_t* __restrict__ fbad, int union_mode) {
    const int b = blockIdx.x, k = threadIdx.x;
    bool acc = true, nonfinite = false, bad = false;
    int tt = -1;
    double my_lse = 0.0, my_lq = 0.0;
    if (k < K) {
        const int64_t row = (int64_t)b * K + k;
        const double lse = combine_parts(part + row * nsplit, nsplit, ratio_t);
        nonfinite = lse != lse;
        my_lse = lse;
        ws_lse_p[row] = lse;
        if (lse_p) lse_p[(int64_t)b * (K + 1) + k] = lse;
        const int d = tok_d[row];
        my_lq = lse_q[row];
        double pd = 0.0, qd = 0.0;
        acc = false;
        // TLI: a draft must be a shared drafter id.  Union algorithm: any drafter id is a legal draft; one
        // outside T has target probability 0 and is rejected by the test itself; every drafter logit takes
        // part there, so a NaN normaliser (NaN/+inf somewhere in the row) flags the sequence.
        if (d < 0 || d >= Vd || (!union_mode && d2t[d] < 0)) {
            bad = true;
        } else if (union_mode && my_lq != my_lq) {
            nonfinite = true;
        } else if (!nonfinite) {
            tt = d2t[d];
            const char* lt = static_cast<const char*>(logits_t) + ((int64_t)b * (K + 1) + k) * Vt * Traits<DT>::ESZ;
            const char* ld = static_cast<const char*>(dv.base) + row * dv.row_stride * Traits<DT>::ESZ;
            pd = (tt < 0 || lse == -INFINITY) ? 0.0 : exp((double)load_elem<DT>(lt, tt) * inv_temp_t - lse);
            const int dx = dv.d2x ? dv.d2x[d] : d;
            qd = (union_mode && my_lq == -INFINITY) ? 0.0 : exp((double)load_elem<DT>(ld, dx) * inv_temp_d - my_lq);
            acc = (double)u_acc[row] * qd < pd;
        }
        if (accept) accept[row] = acc ? 1 : 0;
        if (p_tok) p_tok[row] = pd;
        if (q_tok) q_tok[row] = qd;
    }
    const unsigned long long rej = __ballot(k < K && !acc);
    const bool any_nonfinite = __ballot(nonfinite) != 0ull;
    const bool any_bad = __ballot(bad) != 0ull;
    int n = rej ? (int)__builtin_ctzll(rej) : K;
    if (any_nonfinite) n = 0;
    if (k < K) out_tok[(int64_t)b * (K + 1) + k] = (k < n) ? tt : -1;
    if (k == 0) {
        out_tok[(int64_t)b * (K + 1) + K] = -1;
        n_accepted[b] = n;
        seq_status[b] = (any_nonfinite ? TLI_FLAG_NONFINITE : 0) | (any_bad ? TLI_FLAG_BAD_DRAFT : 0);
        fbad[b] = 0;  // raised by the residual scan if the drafter row it reads holds NaN or +inf
        if (lse_p) lse_p[(int64_t)b * (K + 1) + K] = NAN;
    }
    // one record per sequence for the final kernels, written by the lane that owns the row they will use
    const bool residual = !any_nonfinite && n < K;
    if (residual ? (k == n) : (k == 0)) {
        FinalRow f;
        f.skip = any_nonfinite ? 1 : 0;
        f.bonus = (!any_nonfinite && n == K) ? 1 : 0;
        f.n = n;
        f.t_row = b * (K + 1) + (f.bonus ? K : n);
        f.d_row = b * K + (f.bonus ? 0 : n);
        f.dq = 0.f;
        f.l2p = 0.0;
        f.rp.use_q = 0;
        f.rp.ct_hi = f.rp.ct_lo = f.rp.lp_hi = f.rp.lp_lo = 0.f;
        f.rp.cd_hi = f.rp.cd_lo = f.rp.lq_hi = f.rp.lq_lo = 0.f;
        if (residual) {
            f.l2p = my_lse * kLog2e;
            split_scale(c_t, f.rp.ct_hi, f.rp.ct_lo);
            split_hi_lo(f.l2p, f.rp.lp_hi, f.rp.lp_lo);
            // an unusable draft, or a drafter row without mass, has q' = 0 everywhere
            if (!bad && (my_lq > -INFINITY || my_lq != my_lq)) {
                f.rp.use_q = 1;
                split_scale(c_d, f.rp.cd_hi, f.rp.cd_lo);
                split_hi_lo(my_lq * kLog2e, f.rp.lq_hi, f.rp.lq_lo);
            }
        }
        frow[b] = f;
    }
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

template <int DT>
__device__ __forceinline__ void residual_vec(const void* rowp, int64_t vi, int V, const ResidualParams& rp,
                                             const int32_t* __restrict__ t2d, const void* __restrict__ ld_row,
                                             float* p, float* w) {
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
#pragma unroll
    for (int i = 0; i < EPV; ++i) {
        const bool live = e0 + i < V;
        float pi = exp2_split(x[i], rp.ct_hi, rp.ct_lo, rp.lp_hi, rp.lp_lo);
        pi = live ? pi : 0.f;
        float qi = 0.f;
        if (rp.use_q) {
            qi = exp2_split(y[i], rp.cd_hi, rp.cd_lo, rp.lq_hi, rp.lq_lo);
            qi = (live && d[i] >= 0) ? qi : 0.f;
        }
        p[i] = pi;
        w[i] = fmaxf(0.f, pi - qi);
        if (!(qi <= 3.0e38f)) w[i] = NAN;  // NaN or +inf in the drafter row must surface (fmaxf would drop it)
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

template <int DT>
__device__ __forceinline__ void final_pick_row(const FinalRow& f, int b, const void* logits_t, const DrafterView& dv,
                                               int K, int Vt, int Vd, int nC, float cs_t, double ratio_t,
                                               const int32_t* t2d, const float* tr, const float* ts,
                                               const float2* ctab, const double* mn, const int32_t* fbad,
                                               const FinalOut& o) {
    constexpr int EPV = Traits<DT>::EPV;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const char* rowp = static_cast<const char*>(logits_t) + (int64_t)f.t_row * Vt * Traits<DT>::ESZ;
    const double u = (double)o.u_fin[b];
    int tok = -1;
    int add_flags = 0;
    bool nonfinite = false;
    if (f.bonus) {
        float M;
        double total;
        tok = sample_softmax_row<DT, false>(rowp, Vt, nC, cs_t, ratio_t, nullptr, tr, ts, u, &M, &total);
        // no usable mass: NaN/+inf, or a bonus row of only -inf -- no distribution to sample either way
        if (tok < 0) nonfinite = true;
        else if (threadIdx.x == 0 && o.lse_p) o.lse_p[(int64_t)b * (K + 1) + K] = kLn2 * ((double)M * ratio_t + log2(total));
    } else {
        const char* ldp = static_cast<const char*>(dv.base) + (int64_t)f.d_row * dv.row_stride * Traits<DT>::ESZ;
        // chunk masses: sum_chunk p (from the normaliser kernel's table of row n) minus the parts' sums of min(p, q')
        const float2* crow = ctab + (int64_t)f.d_row * nC;
        auto p_mass = [&](int cc) {
            const float2 rs = crow[cc];
            return (rs.x == -INFINITY) ? 0.0 : (double)rs.y * exp2((double)rs.x * ratio_t - f.l2p);
        };
        auto r_mass = [&](int cc) {
            const double m = f.rp.use_q ? mn[cc] : 0.0;
            const double t = p_mass(cc) - m;
            return t > 0.0 ? t : (t != t ? t : 0.0);
        };
        double theta_local, total;
        int c = -1;
        bool degenerate = false;
        if (f.rp.use_q && fbad[b]) {  // NaN or +inf among the shared drafter logits of row n
            nonfinite = true;
        } else {
            c = find_chunk(nC, u, r_mass, &theta_local, &total);
            if (c < 0) {
                if (total != total) {
                    nonfinite = true;
                } else {  // residual identically zero: fall back to p of the same row
                    degenerate = true;
                    add_flags |= TLI_FLAG_DEGENERATE;
                    c = find_chunk(nC, u, p_mass, &theta_local, &total);
                    if (c < 0) nonfinite = true;
                }
            }
        }
        if (!nonfinite) {
            // wave j of the workgroup takes load j of the chunk: a quarter of the table look-ups, gathers and
            // exponentials each
            const int64_t vi = ((int64_t)c * kLoads + wave) * kWave + lane;
            float p[EPV], w[EPV];
            residual_vec<DT>(rowp, vi, Vt, f.rp, t2d, ldp, p, w);
            double wd[EPV];
#pragma unroll
            for (int i = 0; i < EPV; ++i) wd[i] = degenerate ? (double)p[i] : (double)w[i];
            tok = chunk_draw<EPV>(wd, vi * EPV, theta_local);
        }
    }
    if (threadIdx.x == 0) {
        if (nonfinite) {
            o.n_accepted[b] = 0;
            for (int k = 0; k <= K; ++k) o.out_tok[(int64_t)b * (K + 1) + k] = -1;
            o.seq_status[b] |= TLI_FLAG_NONFINITE;
        } else {
            o.out_tok[(int64_t)b * (K + 1) + f.n] = tok;
            if (add_flags) o.seq_status[b] |= add_flags;
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
constexpr int kScanWG = 1024;
constexpr int kScanWaves = kScanWG / kWave;
constexpr int kSlotBytes = kWave * kLoads * 16;  // one chunk
constexpr int kTrashBytes = kWave * 4;           // LDS [0, 256): a word per lane for the elements a lane does not keep
constexpr int kPartBytes = 92 * 1024;            // then the staged drafter logits of a part, the last 16 bytes of the
                                                 // area hold the -inf logit that padding entries point at
constexpr int kScanLds = kPartBytes + kScanWaves * kSlotBytes;  // then one chunk slot per wave
constexpr int kPairG = 2 * kWave;      // entries in a group of a chunk's pair list: two per lane
constexpr int kPairU = 6;              // groups fetched with a chunk (more: late loop)
constexpr int kStageV = 8;             // drafter vectors a lane has in flight during the staging sweep
constexpr int kPairShift = 16;         // entry = byte offset in chunk (< 4096) | index of the staged logit << 16
constexpr int kMaxPartChunks = kWave * kScanWaves;  // a wave keeps a lane per chunk it handles
static_assert(kScanLds <= 160 * 1024, "LDS of one CU");

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
// pairs a part may hold, and the index of the -inf logit
template <int DT> constexpr int part_cap() { return (kPartBytes - kTrashBytes - 16) / Traits<DT>::ESZ; }
template <int DT> constexpr int dummy_index() { return part_cap<DT>(); }
static_assert(dummy_index<TLI_BF16>() < (1 << 16) && dummy_index<TLI_F32>() < (1 << 16), "16-bit staged index");

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

// DIAG (acceptance-rate diagnostics): the items are all B*K positions instead of one row per sequence, and a
// second sum runs beside the first with the drafter's unrestricted probabilities q = q' * 2^-dq:
// mn = sum min(p, q') (TLI's expected acceptance rate), mn2 = sum min(p, q) (the union algorithm's).
template <int DT, bool DIAG>
__global__ __launch_bounds__(kScanWG) void k_final_scan(
    const void* __restrict__ logits_t, DrafterView dv, int B, int K, int Vt, int Vd, int nC, int nsplit, ScanLists ls,
    float cs_t, double ratio_t, const FinalRow* __restrict__ frow, float* __restrict__ tab_ref, float* __restrict__ tab_s, double* __restrict__ mn, double* __restrict__ mn2,
    int32_t* __restrict__ fbad) {
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
    const FinalRow f = frow[b];
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
        for (int j = 0; j < kLoads; ++j)  // vectors past the row's end re-read its last vector: no pair points there
            r.v[j] = *reinterpret_cast<const u4v*>(trow + min(v0 + j * kWave, (uint32_t)nvec - 1u) * 16u);
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
    double* my_mn = mn + (int64_t)b * nC;
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
        auto two = [&](uint2 e) {
            float u0 = 0.f, u1 = 0.f;
            const float t0 = pair_min(e.x, u0), t1 = pair_min(e.y, u1);
            acc += t0 + t1;
            if (DIAG) acc2 += u0 + u1;
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
        const float tot = wave_sum(acc);
        if (lane == k) keep = (double)tot;
        if (DIAG) {
            const float tot2 = wave_sum(acc2);
            if (lane == k) keep2 = (double)tot2;
        }
    };
    int k = 0;
    for (int idx = gw; idx < ncp; idx += 2 * stride, k += 2) {
        fetch(k + 1, fb);
        process(fa, k);
        fetch(k + 2, fa);
        if (idx + stride < ncp) process(fb, k + 1);
    }
    {
        const int idx = gw + lane * stride;
        if (idx < ncp) {
            my_mn[c_lo + idx] = keep;
            if (DIAG) my_mn2[c_lo + idx] = keep2;
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
                                                       const double* __restrict__ mn,
                                                       const int32_t* __restrict__ fbad, FinalOut o) {
    const int b = blockIdx.x;
    const FinalRow f = frow[b];
    if (f.skip) return;
    final_pick_row<DT>(f, b, logits_t, dv, K, Vt, Vd, nC, cs_t, ratio_t, t2d, tab_ref + (int64_t)b * nC,
                       tab_s + (int64_t)b * nC, ctab, mn + (int64_t)b * nC, fbad, o);
}

// ---- expected acceptance rates of every position ------------------------------------------------
// Table of expected acceptance rates: alpha_union = sum_{T∩D} min{p, q}, alpha_tli = sum_{T∩D} min{p, q'} with
// q' = q / sum_{T∩D} q; the theorem on the intersection algorithm states alpha_union <= alpha_tli.
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
    f.dq = 0.f;
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
        f.dq = (float)((lq2 - lq1) * kLog2e);
    }
    frow[r] = f;
    fbad[r] = 0;
    status[r] = nonfinite ? TLI_FLAG_NONFINITE : (lq1 == -INFINITY ? TLI_FLAG_ZERO_MASS : 0);
}

// kernel: alpha of every position = sum over parts and chunks of the scan's partial sums.  grid (rows), one wave.
__global__ __launch_bounds__(kWave) void k_diag_finish(const FinalRow* __restrict__ frow, const double* __restrict__ mn,
                                                        const double* __restrict__ mn2, int rows, int nC,
                                                        double* __restrict__ alpha_tli, double* __restrict__ alpha_union) {
    const int r = blockIdx.x, lane = threadIdx.x;
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
    if (lane == 0) { alpha_tli[r] = a1; alpha_union[r] = a2; }
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

template <int DT, bool MASKED, bool WHOLE>
__device__ __forceinline__ void chunk_values(const ChunkRegs& r, int c, int lane, int V, const uint64_t* bits, float* x) {
    constexpr int EPV = Traits<DT>::EPV;
    const int64_t v0 = (int64_t)c * (kWave * kLoads) + lane;
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        unpack<DT>(to_uint4(r.v[j]), x + j * EPV);
        const int64_t vi = v0 + j * kWave;
        if (!WHOLE) {
#pragma unroll
            for (int i = 0; i < EPV; ++i)
                if (vi * EPV + i >= V) x[j * EPV + i] = -INFINITY;
        }
        if (MASKED) {
            const uint64_t* w = bits + ((int64_t)c * kLoads + j) * EPV;
#pragma unroll
            for (int i = 0; i < EPV; ++i) {
                const bool keep = __builtin_amdgcn_inverse_ballot_w64(w[i]);
                x[j * EPV + i] = keep ? x[j * EPV + i] : -INFINITY;
            }
        }
    }
}

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
// group, and folded after the scan.  A last pass writes the rows with every dropped logit set to -inf.
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
    int32_t status;
};

// kernel: start the per-row state from the row normalisers.  grid (ceil(R / 256)).
__global__ __launch_bounds__(kWG) void k_warp_init(const Part* __restrict__ part, int nsplit, double ratio, int R,
                                                    int top_k, int use_p, WarpRow* __restrict__ st) {
    const int r = blockIdx.x * kWG + threadIdx.x;
    if (r >= R) return;
    const double lse = combine_parts(part + (int64_t)r * nsplit, nsplit, ratio);
    WarpRow w;
    w.l2 = lse * kLog2e;
    w.zk = 0; w.p_above = 0; w.target = 0; w.kprefix = 0; w.pprefix = 0;
    w.k_rem = top_k > 0 ? (uint32_t)top_k : 0u;
    w.status = lse != lse ? TLI_FLAG_NONFINITE : (lse == -INFINITY ? TLI_FLAG_ZERO_MASS : 0);
    w.k_on = (top_k > 0 && !w.status) ? 1 : 0;
    w.p_on = (use_p && !w.status) ? 1 : 0;
    st[r] = w;
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
    if (MODE == 0 ? !w.k_on : !w.p_on) return;
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
    }
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
    int n = 0;
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
                const bool live = vi * EPV + i < V && ((mb >> i) & 1u) && !w.status && x[i] > -INFINITY &&
                                  (!any || warp_key<DT>(x[i]) >= tkey);
                n += live ? 1 : 0;
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
    for (int d = 1; d < kWave; d <<= 1) n += __shfl_xor(n, d, kWave);
    __shared__ int sn[kWaves];
    if ((threadIdx.x & 63) == 0) sn[threadIdx.x >> 6] = n;
    __syncthreads();
    if (threadIdx.x == 0) {
        int tot = 0;
        for (int i = 0; i < kWaves; ++i) tot += sn[i];
        if (kept) kept[row] = tot;
        if (thr) thr[row] = w.status ? NAN : (any ? warp_unkey<DT>(tkey) : -INFINITY);
        status[row] = w.status;
    }
}

// ---- plain copy, used only to calibrate hardware byte counters against a known size -----------
__global__ __launch_bounds__(kWG) void k_calib_copy(const u4v* __restrict__ src, u4v* __restrict__ dst, size_t nvec) {
    const size_t stride = (size_t)gridDim.x * kWG;
    for (size_t i = (size_t)blockIdx.x * kWG + threadIdx.x; i < nvec; i += stride) dst[i] = src[i];
}

// ======================================= host side ============================================

struct Plan {
    int nC;      // chunks per row
    int nsplit;  // workgroups per row
    int cps;     // chunks per workgroup
};

Plan make_plan(int V, int rows, int chunk) {
    Plan p;
    p.nC = (V + chunk - 1) / chunk;
    const int target_wgs = 2048;  // ~8 workgroups of 4 waves on each of the 256 CUs
    int want = (target_wgs + rows - 1) / rows;
    int cap = (p.nC + kWaves - 1) / kWaves;  // keep at least one chunk per wave
    p.nsplit = want < 1 ? 1 : (want > cap ? cap : want);
    p.cps = (p.nC + p.nsplit - 1) / p.nsplit;
    p.nsplit = (p.nC + p.cps - 1) / p.cps;
    return p;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Workspace {  // offsets into the caller's scratch
    size_t part, part_d, ws_lse_p, ws_lse_q, ctab, frow, fbad, tab_ref, tab_s, mn, total;
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
    w.ws_lse_p = off; off += align256((size_t)rows * sizeof(double));
    w.ws_lse_q = off; off += align256((size_t)rows * sizeof(double));
    w.ctab = off; off += align256((size_t)rows * nCt * sizeof(float2));
    w.frow = off; off += align256((size_t)B * sizeof(FinalRow));
    w.fbad = off; off += align256((size_t)B * sizeof(int32_t));
    w.tab_ref = off; off += align256(tab * sizeof(float));
    w.tab_s = off; off += align256(tab * sizeof(float));
    // the residual scan's sums of min(p, q'), one per chunk of the row the extra token is drawn from
    w.mn = off; off += align256(tab_rows_t * sizeof(double));
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

struct DraftOut;
template <int DT, bool MASKED>
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
    double *ws_lse_p, *ws_lse_q;
    Plan pd;
    float cs_d;
    double ratio_d;
    float *tab_ref, *tab_s;
    double* mn;
    float2* ctab;
    FinalRow* frow;
    int32_t* fbad;
    int union_mode;  // 0: TLI (q' over the shared ids); 1: the union algorithm (q over all of D)
    DrafterView dv;
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


template <int DT, bool MASKED>
void launch_draft(const void* logits, int64_t row_stride, int R, int V, float temp, const Plan& pl, float cs,
                  double ratio, const uint64_t* bits, const int32_t* d2t, const DraftOut& o, float* tab_ref,
                  float* tab_s, hipStream_t st) {
    const double inv_temp = 1.0 / (double)temp;
    if (pl.nsplit == 1 && pl.nC <= kLdsChunks) {  // enough rows to fill the chip with one workgroup per row
        KernelTimer t(TLI_KERNEL_DRAFT_SCAN, st);
        hipLaunchKernelGGL((k_draft_fused<DT, MASKED>), dim3(R), dim3(kWG), 0, st, logits, row_stride, V, pl.nC, cs, ratio,
                           inv_temp, bits, d2t, o);
        return;
    }
    {
        KernelTimer t(TLI_KERNEL_DRAFT_SCAN, st);
        hipLaunchKernelGGL((k_draft_scan<DT, MASKED>), dim3((unsigned)R * pl.nsplit), dim3(kWG), 0, st, logits, row_stride,
                           V, pl.nC, pl.cps, pl.nsplit, cs, ratio, bits, tab_ref, tab_s);
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
                     const int32_t* r2d = nullptr) {
    if (!logits || !u || !tok || !status || !workspace) return TLI_ERR_INVALID_ARG;
    if (R < 1 || R > 0x7fffffff / 64 || V < 1 || !(temp > 0.f) || !std::isfinite(temp) || io_stride < 1)
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
    if (R < 1 || R > 0x7fffffff / 64 || V < 1 || io_stride < 1) return TLI_ERR_INVALID_ARG;
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

template <int DT> void launch_verify(const VerifyArgs& a, hipStream_t st) {
    const int Vt = a.map->Vt, Vd = a.map->Vd, B = a.B, K = a.K, rows = B * K;
    FinalOut fo;
    fo.u_fin = a.u_fin; fo.n_accepted = a.n_accepted; fo.out_tok = a.out_tok; fo.lse_p = a.lse_p;
    fo.seq_status = a.seq_status;
    const double* lse_q = a.lse_q;
    if (!lse_q) {  // the caller did not keep the drafter normalisers: one scan of the drafter rows (masked for TLI
                   // in the full layout; a compact row holds the shared ids only)
        const int64_t rs = a.dv.row_stride;
        if (a.union_mode || a.compact)
            hipLaunchKernelGGL((k_lse<DT, false>), dim3((unsigned)rows * a.pd.nsplit), dim3(kWG), 0, st, a.dv.base, K,
                               (int64_t)K * rs, rs, a.d_valid, a.pd.nC, a.pd.cps, a.pd.nsplit, a.cs_d, a.ratio_d,
                               (const uint64_t*)nullptr, a.part_d, (float2*)nullptr);
        else
            hipLaunchKernelGGL((k_lse<DT, true>), dim3((unsigned)rows * a.pd.nsplit), dim3(kWG), 0, st, a.dv.base, K,
                               (int64_t)K * rs, rs, a.d_valid, a.pd.nC, a.pd.cps, a.pd.nsplit, a.cs_d, a.ratio_d,
                               a.map->lmask[DT], a.part_d, (float2*)nullptr);
        hipLaunchKernelGGL(k_lse_finish, dim3((rows + kWG - 1) / kWG), dim3(kWG), 0, st, a.part_d, rows, a.pd.nsplit,
                           a.ratio_d, a.ws_lse_q);
        lse_q = a.ws_lse_q;
    }
    {
        KernelTimer t(TLI_KERNEL_LSE, st);
        hipLaunchKernelGGL((k_lse<DT, false>), dim3((unsigned)rows * a.pl.nsplit), dim3(kWG), 0, st, a.logits_t, K,
                           (int64_t)(K + 1) * Vt, (int64_t)Vt, Vt, a.pl.nC, a.pl.cps, a.pl.nsplit, a.cs_t, a.ratio_t,
                           nullptr, a.part, a.ctab);
    }
    {
        KernelTimer t(TLI_KERNEL_ACCEPT, st);
        hipLaunchKernelGGL(k_accept<DT>, dim3(B), dim3(kWave), 0, st, a.logits_t, a.dv, K, Vt, Vd, a.pl.nsplit,
                           a.part, a.ratio_t, a.inv_t, a.inv_d, a.map->d2t, a.tok_d, lse_q, a.u_acc, a.n_accepted,
                           a.out_tok, a.accept, a.p_tok, a.q_tok, a.lse_p, a.seq_status, a.ws_lse_p, a.c_t, a.c_d, a.frow,
                           a.fbad, a.union_mode);
    }
    {
        KernelTimer t(TLI_KERNEL_FINAL_SCAN, st);
        const int nparts = a.map->scan[DT].nparts;
        // few sequences: deal the chunks of a (sequence, part) to several workgroups, up to one per CU
        int nsplit = 256 / (B * nparts);
        nsplit = nsplit < 1 ? 1 : (nsplit > 4 ? 4 : nsplit);
        const ScanLists ls = scan_lists(a.map, DT, a.compact ? 1 : 0);
        hipLaunchKernelGGL((k_final_scan<DT, false>), dim3((unsigned)((B + 7) / 8) * 8 * nparts * nsplit), dim3(kScanWG), 0,
                           st, a.logits_t, a.dv, B, K, Vt, Vd, a.pf.nC, nsplit, ls, a.cs_t, a.ratio_t, a.frow, a.tab_ref,
                           a.tab_s, a.mn, (double*)nullptr, a.fbad);
    }
    {
        KernelTimer t(TLI_KERNEL_FINAL_PICK, st);
        hipLaunchKernelGGL(k_final_pick<DT>, dim3(B), dim3(kLoads * kWave), 0, st, a.logits_t, a.dv, K, Vt, Vd, a.pf.nC,
                           a.cs_t, a.ratio_t, a.frow, a.dv.t2x, a.tab_ref, a.tab_s, a.ctab, a.mn, a.fbad, fo);
    }
}

}  // namespace

namespace {
struct DiagLayout { size_t part_t, part_q1, part_q2, frow, fbad, mn, mn2, total; };
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
    hipLaunchKernelGGL((k_lse<DT, false>), dim3((unsigned)rows * pt.nsplit), dim3(kWG), 0, st, logits_t, K,
                       (int64_t)(K + 1) * Vt, (int64_t)Vt, Vt, pt.nC, pt.cps, pt.nsplit, cs_t, ratio_t,
                       (const uint64_t*)nullptr, part_t, (float2*)nullptr);
    hipLaunchKernelGGL((k_lse<DT, true>), dim3((unsigned)rows * pd.nsplit), dim3(kWG), 0, st, logits_d, K, (int64_t)K * Vd,
                       (int64_t)Vd, Vd, pd.nC, pd.cps, pd.nsplit, cs_d, ratio_d, map->lmask[DT], part_q1, (float2*)nullptr);
    hipLaunchKernelGGL((k_lse<DT, false>), dim3((unsigned)rows * pd.nsplit), dim3(kWG), 0, st, logits_d, K, (int64_t)K * Vd,
                       (int64_t)Vd, Vd, pd.nC, pd.cps, pd.nsplit, cs_d, ratio_d, (const uint64_t*)nullptr, part_q2,
                       (float2*)nullptr);
    hipLaunchKernelGGL(k_diag_rows, dim3((rows + kWG - 1) / kWG), dim3(kWG), 0, st, part_t, pt.nsplit, part_q1, part_q2,
                       pd.nsplit, rows, K, ratio_t, ratio_d, c_t, c_d, frow, fbad, status);
    const int nparts = map->scan[DT].nparts;
    int nsplit = 256 / (rows * nparts);
    nsplit = nsplit < 1 ? 1 : (nsplit > 4 ? 4 : nsplit);
    const ScanLists ls = scan_lists(map, DT, 0);
    hipLaunchKernelGGL((k_final_scan<DT, true>), dim3((unsigned)((rows + 7) / 8) * 8 * nparts * nsplit), dim3(kScanWG), 0, st,
                       logits_t, DrafterView{logits_d, (int64_t)Vd, nullptr, map->t2d}, rows, K, Vt, Vd, pt.nC, nsplit, ls,
                       cs_t, ratio_t, frow, (float*)nullptr, (float*)nullptr, mn, mn2, fbad);
    hipLaunchKernelGGL(k_diag_finish, dim3(rows), dim3(kWave), 0, st, frow, mn, mn2, rows, pt.nC, alpha_tli,
                       alpha_union);
}
}  // namespace

extern "C" {

int tli_calib_copy(const void* src, void* dst, size_t bytes, void* hip_stream) {
    if (!src || !dst || bytes == 0 || bytes % 16 != 0 || !aligned16(src) || !aligned16(dst)) return TLI_ERR_INVALID_ARG;
    hipLaunchKernelGGL(k_calib_copy, dim3(4096), dim3(kWG), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const u4v*>(src), static_cast<u4v*>(dst), bytes / 16);
    return hipGetLastError() == hipSuccess ? TLI_OK : TLI_ERR_HIP;
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
        default: return "TLI_ERR_UNKNOWN";
    }
}

int tli_build_map(const int32_t* d2t_host, int32_t Vd, int32_t Vt, tli_map** out_map, int32_t* out_num_shared) {
    if (out_map) *out_map = nullptr;
    if (out_num_shared) *out_num_shared = 0;
    if (!d2t_host || !out_map || Vd < 1 || Vt < 1) return TLI_ERR_INVALID_ARG;
    const size_t Vd_pad = ((size_t)Vd + 7) & ~(size_t)7, Vt_pad = ((size_t)Vt + 7) & ~(size_t)7;
    std::vector<int32_t> d2t(Vd_pad, -1), t2d(Vt_pad, -1);
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
    // rank -> drafter id, and per dtype the pair lists of the residual scan (see tli_map)
    std::vector<int32_t> sh_x(S);
    {
        int32_t r = 0;
        for (int32_t x = 0; x < Vd; ++x)
            if (d2t[x] >= 0) sh_x[r++] = x;
    }
    struct HostScan {
        std::vector<int32_t> cb, part_n, pl_g;
        int NV[2];
        std::vector<uint32_t> stab[2];
        std::vector<int2> grange[2];
        std::vector<uint2> pl_e[2];
    } hs[2];
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
        for (int p = 0; p < nparts; ++p)
            for (int c = h.cb[p]; c < h.cb[p + 1]; ++c) { part_of_chunk[c] = p; h.part_n[p] += cc[c]; }
        h.pl_g.assign(nC + 1, 0);
        for (int c = 0; c < nC; ++c) h.pl_g[c + 1] = h.pl_g[c] + (cc[c] + kPairG - 1) / kPairG;
        for (int layout = 0; layout < 2; ++layout) {
            // staging table: what the sweep over a drafter row (element index = drafter id in the full layout,
            // rank in the compact one) keeps of every vector for a part, and where it puts it
            const int64_t elems = layout ? S : Vd;
            const int NV = (int)(((elems + epv - 1) / epv + kWave - 1) / kWave) * kWave;
            h.NV[layout] = NV;
            h.stab[layout].assign((size_t)nparts * NV, 0);
            h.grange[layout].assign(nparts, make_int2(NV / kWave, 0));
            for (int32_t r = 0; r < S; ++r) {
                const int64_t x = layout ? r : sh_x[r];
                const int p = part_of_chunk[d2t[sh_x[r]] / CH];
                h.stab[layout][(size_t)p * NV + x / epv] |= 1u << (16 + x % epv);
                const int g = (int)(x / epv / kWave);
                if (g < h.grange[layout][p].x) h.grange[layout][p].x = g;
                if (g + 1 > h.grange[layout][p].y) h.grange[layout][p].y = g + 1;
            }
            for (int p = 0; p < nparts; ++p) {
                if (h.grange[layout][p].y == 0) h.grange[layout][p] = make_int2(0, 0);  // a part without pairs
                uint32_t run = 0;
                for (int vi = 0; vi < NV; ++vi) {
                    uint32_t& w = h.stab[layout][(size_t)p * NV + vi];
                    const uint32_t cnt = (uint32_t)__builtin_popcount(w >> 16);
                    w |= cnt ? run : 0;  // vectors that keep nothing never use the index
                    run += cnt;
                }
            }
            // pairs grouped by target chunk (ranks ascending inside a chunk): entry n of a chunk's list sits in
            // group n / kPairG, lane n % 64, first or second of the lane's two by (n % kPairG) / 64
            const uint32_t dummy = (uint32_t)(dt == TLI_BF16 ? dummy_index<TLI_BF16>() : dummy_index<TLI_F32>()) << kPairShift;
            h.pl_e[layout].assign(((size_t)h.pl_g[nC] + kPairU) * kWave, make_uint2(dummy, dummy));
            std::vector<int32_t> nth(nC, 0);
            for (int32_t r = 0; r < S; ++r) {
                const int64_t x = layout ? r : sh_x[r];
                const int32_t t = d2t[sh_x[r]];
                const int c = t / CH, p = part_of_chunk[c];
                const uint32_t w = h.stab[layout][(size_t)p * NV + x / epv];
                const uint32_t pos = (w & 0xffffu) + (uint32_t)__builtin_popcount((w >> 16) & ((1u << (x % epv)) - 1u));
                const uint32_t e = (uint32_t)(t % CH) * esz | (pos << kPairShift);
                const int n = nth[c]++;
                uint2& slot = h.pl_e[layout][((size_t)h.pl_g[c] + n / kPairG) * kWave + n % kWave];
                if ((n % kPairG) / kWave == 0) slot.x = e; else slot.y = e;
            }
        }
    }
    // shared-id mask of the drafter vocabulary in lane-mask layout (see mask_bits), padded to whole chunks
    std::vector<uint64_t> lmask[2];
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
    tli_map* m = new (std::nothrow) tli_map();
    if (!m) return TLI_ERR_ALLOC;
    m->Vd = Vd; m->Vt = Vt; m->S = S; m->d2t = nullptr; m->t2d = nullptr; m->lmask[0] = m->lmask[1] = nullptr;
    m->sh_x = nullptr; m->d2r = nullptr; m->t2r = nullptr;
    for (int dt = 0; dt < 2; ++dt) {
        tli_map::Scan& sc = m->scan[dt];
        sc.nparts = (int32_t)hs[dt].part_n.size();
        sc.cb = sc.part_n = sc.pl_g = nullptr;
        for (int layout = 0; layout < 2; ++layout) {
            sc.NV[layout] = hs[dt].NV[layout];
            sc.stab[layout] = nullptr; sc.grange[layout] = nullptr; sc.pl_e[layout] = nullptr;
        }
    }
    if (hipGetDevice(&m->device) != hipSuccess) { delete m; return TLI_ERR_HIP; }
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
            {(void**)&sc.grange[0], h.grange[0].data(), h.grange[0].size() * sizeof(int2)},
            {(void**)&sc.grange[1], h.grange[1].data(), h.grange[1].size() * sizeof(int2)},
            {(void**)&sc.pl_e[0], h.pl_e[0].data(), h.pl_e[0].size() * sizeof(uint2)},
            {(void**)&sc.pl_e[1], h.pl_e[1].data(), h.pl_e[1].size() * sizeof(uint2)},
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
    if (B < 1 || K < 1 || K > kMaxK || Vt < 1 || Vd < 1 || (dtype != TLI_F32 && dtype != TLI_BF16)) return 0;
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
    if (R < 1 || R > 0x7fffffff / 64 || V < 1 || (dtype != TLI_F32 && dtype != TLI_BF16)) return 0;
    const int chunk = dtype == TLI_BF16 ? chunk_elems<TLI_BF16>() : chunk_elems<TLI_F32>();
    const Plan pl = make_plan(V, R, chunk);
    return align256((size_t)R * pl.nsplit * sizeof(Part)) + align256((size_t)R * sizeof(WarpRow));
}

int tli_warp_rows(const tli_map* map, const void* logits, tli_dtype dtype, int64_t row_stride_elems, int32_t R, int32_t V,
                  float temp, int32_t top_k, float top_p, void* logits_out, int64_t out_stride_elems, float* thr,
                  int32_t* kept, int32_t* row_status, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!logits || !logits_out || !row_status || !workspace) return TLI_ERR_INVALID_ARG;
    if (R < 1 || R > 0x7fffffff / 64 || V < 1 || !(temp > 0.f) || !std::isfinite(temp)) return TLI_ERR_INVALID_ARG;
    if (!(top_p > 0.f) || (map && V != map->Vd)) return TLI_ERR_INVALID_ARG;
    if (dtype != TLI_F32 && dtype != TLI_BF16) return TLI_ERR_INVALID_ARG;
    const int epv = dtype == TLI_BF16 ? 8 : 4;
    if (row_stride_elems < V || row_stride_elems % epv != 0 || out_stride_elems < V || out_stride_elems % epv != 0 ||
        !aligned16(logits) || !aligned16(logits_out) || !aligned16(workspace))
        return TLI_ERR_INVALID_ARG;
    if (workspace_bytes < tli_warp_workspace_bytes(R, V, dtype)) return TLI_ERR_ALLOC;
    const int chunk = dtype == TLI_BF16 ? chunk_elems<TLI_BF16>() : chunk_elems<TLI_F32>();
    const Plan pl = make_plan(V, R, chunk);
    Part* part = reinterpret_cast<Part*>(workspace);
    WarpRow* st = reinterpret_cast<WarpRow*>(static_cast<char*>(workspace) + align256((size_t)R * pl.nsplit * sizeof(Part)));
    const double c_true = kLog2e / (double)temp;
    const float cs = (float)c_true;
    const double ratio = c_true / (double)cs;
    const int use_p = top_p < 1.f ? 1 : 0;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const dim3 rows_grid(R), lse_grid((unsigned)R * pl.nsplit);
#define TLI_WARP_RUN(DT, MASKED, BITS)                                                                                   \
    do {                                                                                                                  \
        hipLaunchKernelGGL((k_lse<DT, MASKED>), lse_grid, dim3(kWG), 0, s, logits, 1, row_stride_elems, row_stride_elems, \
                           V, pl.nC, pl.cps, pl.nsplit, cs, ratio, BITS, part, (float2*)nullptr);                        \
        hipLaunchKernelGGL(k_warp_init, dim3((R + kWG - 1) / kWG), dim3(kWG), 0, s, part, pl.nsplit, ratio, R, top_k,     \
                           use_p, st);                                                                                    \
        if (top_k > 0)                                                                                                    \
            for (int level = 0; level < WarpKey<DT>::LEVELS; ++level)                                                     \
                hipLaunchKernelGGL((k_warp_level<DT, MASKED, 0>), rows_grid, dim3(kWG), 0, s, logits, row_stride_elems,   \
                                   V, pl.nC, level, top_p, c_true, BITS, st);                                             \
        if (use_p)                                                                                                        \
            for (int level = 0; level < WarpKey<DT>::LEVELS; ++level)                                                     \
                hipLaunchKernelGGL((k_warp_level<DT, MASKED, 1>), rows_grid, dim3(kWG), 0, s, logits, row_stride_elems,   \
                                   V, pl.nC, level, top_p, c_true, BITS, st);                                             \
        hipLaunchKernelGGL((k_warp_apply<DT, MASKED>), rows_grid, dim3(kWG), 0, s, logits, row_stride_elems, V, pl.nC,    \
                           BITS, st, logits_out, out_stride_elems, thr, kept, row_status);                                \
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
    if (R < 1 || R > 0x7fffffff / 64 || V < 1 || (dtype != TLI_F32 && dtype != TLI_BF16)) return 0;
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
    if (B < 1 || m < 1 || m >= kMaxK || (int64_t)B * (m + 1) > 0x7fffffff / 64 || Vt < 1) return TLI_ERR_INVALID_ARG;
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
    if (B < 1 || m < 1 || m >= kMaxK || (int64_t)B * (m + 1) > 0x7fffffff / 64 || Vt < 1 ||
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
    double* ws_lse_p = reinterpret_cast<double*>(ws + w.ws_lse_p);
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
    a.seq_status = seq_status; a.part = part; a.ws_lse_p = ws_lse_p;
    a.part_d = reinterpret_cast<Part*>(ws + w.part_d); a.ws_lse_q = reinterpret_cast<double*>(ws + w.ws_lse_q);
    a.compact = compact ? 1 : 0;
    a.d_valid = compact ? map->S : Vd;
    a.dv.base = logits_d;
    a.dv.row_stride = compact ? compact_stride : (int64_t)Vd;
    a.dv.d2x = compact ? map->d2r : nullptr;
    a.dv.t2x = compact ? map->t2r : map->t2d;
    a.pd = make_plan(a.d_valid, rows, chunk); a.cs_d = (float)c_d; a.ratio_d = c_d / (double)a.cs_d; a.tab_ref = tab_ref; a.tab_s = tab_s;
    a.mn = reinterpret_cast<double*>(ws + w.mn); a.fbad = reinterpret_cast<int32_t*>(ws + w.fbad); a.ctab = reinterpret_cast<float2*>(ws + w.ctab);
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
