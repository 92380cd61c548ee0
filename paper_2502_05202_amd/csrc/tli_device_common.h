// tli_device_common.h -- Constants, storage traits, wave64 reductions, chunk loads and the per-chunk reduction that every kernel of the
// path is built from.  Included by tli_kernels.hip inside its unnamed namespace (after tli_layout.h, whose names --
// kWave, kLoads, Traits, chunk_elems -- are in scope there).
#pragma once

constexpr int kWG = 256;
constexpr int kWaves = kWG / kWave;
constexpr int kMaxK = 64;
constexpr int kLdsChunks = 1024;  // chunk-table entries a workgroup may park in LDS
constexpr double kLn2 = 0.693147180559945309417232121458;
constexpr double kLog2e = 1.44269504088896340735992468100;

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

// The logits of a chunk held in registers, as floats: x[j * EPV + i] = element i of load j; ids past the vocabulary and
// (MASKED) ids not marked in `bits` read as -inf.
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

// Reduce one chunk held in registers to (ref, s): sum 2^(x*c) over the chunk = s * 2^ref, with
// ref = ceil(max over the chunk of fp32(x*c)) (-inf and s = 0 for a chunk without finite entries).
// A NaN or +inf logit turns s into NaN.  Wave-uniform results.  WHOLE: every element is < V.
// MASKED: bit 0 = only the ids marked in `bits` take part; bit 1 = only logits >= thr do (a warped row, given by
// its threshold instead of rewritten; a NaN logit still shows).
template <int DT, int MASKED, bool WHOLE>
__device__ __forceinline__ void reduce_chunk(const ChunkRegs& r, int c, int lane, int V, float cs, float dl,
                                             const uint64_t* bits, float& ref_out, float& s_out,
                                             float thr = -INFINITY) {
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
        if (MASKED & 1) {
            const uint64_t* w = bits + ((int64_t)c * kLoads + j) * EPV;  // wave-uniform address: scalar loads
#pragma unroll
            for (int i = 0; i < EPV; ++i) {
                const bool keep = __builtin_amdgcn_inverse_ballot_w64(w[i]);
                x[j * EPV + i] = keep ? x[j * EPV + i] : -INFINITY;
            }
        }
        if (MASKED & 2) {
#pragma unroll
            for (int i = 0; i < EPV; ++i) x[j * EPV + i] = x[j * EPV + i] < thr ? -INFINITY : x[j * EPV + i];
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
    // (a lane whose largest logit is -inf: its sum is 0 as it stands -- or NaN, if a NaN sits among its -inf
    // logits, which the maximum does not see and which must surface)
    s = (m == -INFINITY) ? s : s * exp2_hw(fmaf(e, dl, e));
    ref_out = R;
    s_out = wave_sum(s);
}

// reduce_chunk's arithmetic on values that are already unpacked (and masked): for kernels that look at the values
// themselves as well
template <int N>
__device__ __forceinline__ void reduce_values(const float* x, float cs, float dl, float& ref_out, float& s_out) {
    float m = x[0];
#pragma unroll
    for (int i = 1; i < N; ++i) m = fmaxf(m, x[i]);
    const float ref = m * cs;
    const float nref = (m == -INFINITY) ? 0.f : -ref;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i & 3] += exp2_hw(fmaf(x[i], cs, nref));
    float s = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    const float R = ceilf(wave_max(ref));
    const float e = ref - R;
    // (a lane whose largest logit is -inf: its sum is 0 as it stands -- or NaN, if a NaN sits among its -inf
    // logits, which the maximum does not see and which must surface)
    s = (m == -INFINITY) ? s : s * exp2_hw(fmaf(e, dl, e));
    ref_out = R;
    s_out = wave_sum(s);
}

// The same reduction for two sums at once -- over every id of the chunk (s_all) and over the shared ids only
// (s_sh) -- with one exponential per logit: both are formed against the lane's maximum over ALL its ids and leave
// with the chunk reference of the full sum.  That is only as accurate as a reduction of the shared ids alone while
// the shared maximum of the chunk lies within 2^64 of the full one (the shared terms that matter then stay normal
// fp32 numbers); `ok` (wave-uniform) says so, and is false as well for a chunk without shared mass or with a +inf
// or NaN maximum: the caller then reduces the shared ids on their own.
template <int DT, bool WHOLE>
__device__ __forceinline__ void reduce_chunk_both(const ChunkRegs& r, int c, int lane, int V, float cs, float dl,
                                                  const uint64_t* bits, float& ref_out, float& s_all_out,
                                                  float& s_sh_out, bool& ok) {
    constexpr int EPV = Traits<DT>::EPV;
    constexpr int N = EPV * kLoads;
    float x[N];
    const int64_t v0 = (int64_t)c * (kWave * kLoads) + lane;
    float m = -INFINITY, msh = -INFINITY;
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        unpack<DT>(to_uint4(r.v[j]), x + j * EPV);
        const int64_t vi = v0 + j * kWave;
        const uint64_t* w = bits + ((int64_t)c * kLoads + j) * EPV;  // wave-uniform address: scalar loads
#pragma unroll
        for (int i = 0; i < EPV; ++i) {
            if (!WHOLE && vi * EPV + i >= V) x[j * EPV + i] = -INFINITY;
            const bool keep = __builtin_amdgcn_inverse_ballot_w64(w[i]);
            m = fmaxf(m, x[j * EPV + i]);
            msh = fmaxf(msh, keep ? x[j * EPV + i] : -INFINITY);
        }
    }
    const float ref = m * cs;  // the rounded product that the fma below subtracts (see reduce_chunk)
    const float nref = (m == -INFINITY) ? 0.f : -ref;
    float acc[4] = {0.f, 0.f, 0.f, 0.f}, ash[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < kLoads; ++j) {
        const uint64_t* w = bits + ((int64_t)c * kLoads + j) * EPV;
#pragma unroll
        for (int i = 0; i < EPV; ++i) {
            const float e = exp2_hw(fmaf(x[j * EPV + i], cs, nref));
            const bool keep = __builtin_amdgcn_inverse_ballot_w64(w[i]);
            acc[i & 3] += e;
            ash[i & 3] += keep ? e : 0.f;
        }
    }
    const float rmax = wave_max(ref), rsh = wave_max(msh * cs);
    ok = rmax < INFINITY && rsh > -INFINITY && rmax - rsh <= 64.f;
    const float R = ceilf(rmax);
    const float e = ref - R;
    const float f = (m == -INFINITY) ? 0.f : exp2_hw(fmaf(e, dl, e));
    ref_out = R;
    // (largest logit -inf: the sums are 0 as they stand, or NaN if a NaN sits among the lane's -inf logits)
    const float sa = (acc[0] + acc[1]) + (acc[2] + acc[3]), ss = (ash[0] + ash[1]) + (ash[2] + ash[3]);
    s_all_out = wave_sum((m == -INFINITY) ? sa : sa * f);
    s_sh_out = wave_sum((m == -INFINITY) ? ss : ss * f);
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
template <int DT, int MASKED, int NW, class Sink>
__device__ __forceinline__ void scan_chunks(const u4v* rowv, int V, int c_begin, int c_end, float cs, float dl,
                                            const uint64_t* bits, Sink&& sink, float thr = -INFINITY) {
    const int lane = threadIdx.x & 63;
    stream_chunks<DT, NW>(rowv, V, c_begin, c_end, [&](const ChunkRegs& r, int c, auto whole) {
        float ref, sum;
        reduce_chunk<DT, MASKED, decltype(whole)::value>(r, c, lane, V, cs, dl, bits, ref, sum, thr);
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
        if (nr == -INFINITY) { s += (double)sc; return; }  // sc is 0 -- or NaN (a NaN among -inf logits), which must stay
        s = s * exp2_diff(ref, nr, kd) + (double)sc * exp2_diff(r, nr, kd);
        ref = nr;
    }
};

struct Part {  // partial log-normaliser of (a split of) a row: sum 2^(x*c) = s * 2^ref
    float ref;
    float pad;
    double s;
};
