// SpecSteer verify-and-recover block for MI355X (gfx950): HIP kernels and the C ABI.
//
// What is computed (Algorithm 1 phases 2-3, Eq. 7, Eq. 8) is stated in
// include/specsteer.h.  How it is computed here:
//
//   row_lse        the dominant, HBM-bound pass.  Every valid row of G and S_noctx is
//                  cut into slices; one 64-lane wavefront streams one slice with
//                  non-temporal 16-byte loads and keeps a per-lane running (E, s) with
//                  sum_v 2^(h_v*c - E) = s,  c = log2(e)/T,  E an integer >= max(h*c).
//                  An integer reference makes every rescale an exact ldexp and costs
//                  no extra exponential: one v_exp_f32 per logit.  Waves never
//                  synchronise with each other (no barrier in the loop); a persistent
//                  grid strides over the slice list.  A ragged batch's row list is an
//                  exclusive scan of the draft lengths that every workgroup rebuilds in
//                  LDS at kernel start (prep_rows does it once in global memory for
//                  batches too large for LDS).
//   accept_recover one 16-wave workgroup per sequence.  Each (position, tensor) pair
//                  gets a lane that merges the row's slice partials and gathers the draft
//                  token's logit; wave 0 applies the ratio test and finds the first
//                  rejection with a ballot.  All waves then stream the three logit rows
//                  of the rejected (or bonus) position once, forming the recovery
//                  exponent in double (in fp32, as the row pass does, when beta == 0 leaves
//                  no steering term), and record one (E, s) mass per 2048-logit chunk
//                  in LDS.  A double-precision scan over the chunk masses locates the
//                  chunk holding u*Z; only that chunk is read again to pick the token.
//                  The full log-prob row is a second sweep, taken only on request.
//                  Batches of at most 128 sequences share each recovery row between
//                  several workgroups; the one that delivers its chunk masses last
//                  draws the token (see accept_recover_kernel; hand-over by write-through
//                  stores and an arrival counter, without cache-wide fences).
//
// Precision: logits are widened exactly; sums of exponentials are accumulated in
// fp32 (one rounding per term, pairwise across lanes), every per-row scalar
// (log-sum-exp combine, log-probs, alpha, CDF walk across chunks) is double.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "device_common.h"
#include "specsteer.h"

namespace {

constexpr int kLseThreads = 256;            // 4 independent waves per workgroup
// Launch-shape constants of the row pass; the defaults are the measured optimum on MI355X for
// the B=256, V=128256 bf16 workload and can be overridden at build time for other sweeps.
#ifndef SS_LSE_UNROLL
#define SS_LSE_UNROLL 4
#endif
#ifndef SS_LSE_WG_PER_CU
#define SS_LSE_WG_PER_CU 4
#endif
#ifndef SS_LSE_MAX_SLICE_VECS
#define SS_LSE_MAX_SLICE_VECS 4096
#endif
constexpr int kLseUnroll = SS_LSE_UNROLL;   // 16-byte loads in flight per lane
constexpr int kLseWgPerCu = SS_LSE_WG_PER_CU;  // persistent workgroups per CU
constexpr int kMinSliceVecs = kWave * kLseUnroll;  // smallest slice: one unrolled group
constexpr int kMaxSliceVecs = SS_LSE_MAX_SLICE_VECS;  // 64 KiB of logits per slice
constexpr int kMaxSlices = 64;
constexpr int kMaxLdsBatch = 8192;          // ragged batches up to this size keep their row list in LDS
constexpr int kChunkSteps = 4;              // recovery chunk = 4 wave-steps (2048 bf16 logits)
constexpr int kEInit = -(1 << 29);          // "no logit seen yet" exponent reference
constexpr float kEClamp = 5.0e8f;           // keeps (int)ceil(h*c) inside int32 for any finite h
constexpr double kLn2 = 0.693147180559945309417232121458;
constexpr double kLog2e = 1.442695040888963407359924681002;

constexpr int kRecThreads = 1024;           // accept + recover: one 16-wave workgroup per sequence ...
constexpr int kRecThreadsHalf = 512;        // ... or two 8-wave workgroups per CU when sequences outnumber the CUs

struct Partial {
    int E;    // integer exponent reference of this slice
    float s;  // sum over the slice of 2^(h*c - E)
};

// ------------------------------------------------------------------ online sum of exponentials

struct Acc {
    int E;
    float s;
};

__device__ __forceinline__ int exp_ref(float scaled_max) {
    return (int)ceilf(fminf(fmaxf(scaled_max, -kEClamp), kEClamp));
}

// fp32 path of the row pass: term = 2^(h*c_hi - E), c_hi = fl32(c).  The rounding of c would cost
// |h/T| * 2^-24 in the log-sum; it is repaid when the partials are merged: with z = h*c_hi - E
// the missing factor is 2^((z + E)*rho), rho = (c - c_hi)/c_hi ~ 2^-25, and the terms that carry
// the sum have |z| of a few units, so adding E*rho to the row's log2-sum leaves ~|z|*rho < 1e-6.
template <int N>
__device__ __forceinline__ void acc_add_f32(Acc& a, const float (&h)[N], float c_hi) {
    float m = h[0];
#pragma unroll
    for (int i = 1; i < N; ++i) m = fmaxf(m, h[i]);
    const int En = max(a.E, exp_ref(m * c_hi));
    a.s = ldexpf(a.s, a.E - En);
    a.E = En;
    const float nE = -(float)En;
    float t0 = 0.f, t1 = 0.f;
#pragma unroll
    for (int i = 0; i < N; i += 2) {
        t0 += __builtin_amdgcn_exp2f(fmaf(h[i], c_hi, nE));
        if (i + 1 < N) t1 += __builtin_amdgcn_exp2f(fmaf(h[i + 1], c_hi, nE));
    }
    a.s += t0 + t1;
}

// The steering difference h_SLM^+ - h_SLM^- of Eq. 8.  A token masked (-inf) in both specialist rows
// carries no steering -- 0, not inf - inf; for equal finite logits the result is the same 0 as before.
__device__ __forceinline__ float steer_diff(float sp, float sm) { return sp == sm ? 0.f : sp - sm; }
__device__ __forceinline__ double steer_diff_d(float sp, float sm) { return sp == sm ? 0.0 : (double)sp - (double)sm; }

// recovery logit in the base-2 exponent domain: y = (G + beta*(S_ctx - S_noctx)) * log2(e)/T, in double.
__device__ __forceinline__ double rec_y(float g, float sp, float sm, double c, double bc) {
    return fma((double)g, c, steer_diff_d(sp, sm) * bc);
}

// Recovery pass accumulate.  The exponent reference is advanced from a cheap fp32 estimate of
// this vector's maximum; the term exponents themselves are formed in double,
//     z = g*c + (sp - sm)*beta*c - E   (two fused multiply-adds, E folded into the first),
// so the only roundings are the final conversion of the small number z to fp32 and the
// exponential.  sp - sm is taken in fp32: exact for bf16 inputs whose exponents differ by
// less than 16 (otherwise the smaller one is below 2^-16 of the larger and the difference
// rounds by at most 2^-25 of it); fp32 inputs widen first.
// Greedy decoding needs argmax of Eq. 8 itself: h_LLM + beta*(h_SLM^+ - h_SLM^-) as one exact
// difference, one rounded product and one rounded sum in double -- the same three operations
// the definition spells out, so the winner is reproducible bit for bit.  Strict '>' keeps the
// lowest index, because a lane meets its logits in increasing vocabulary order.
struct Best {
    double v;
    long idx;
};

template <int DT, int N, bool GREEDY>
__device__ __forceinline__ void acc_add_rec(Acc& a, const float (&hg)[N], const float (&hp)[N], const float (&hm)[N],
                                            double c, double bc, float cf, float bcf, double beta, long first,
                                            Best& best) {
    if (GREEDY) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const double hr = __dadd_rn((double)hg[i], __dmul_rn(beta, steer_diff_d(hp[i], hm[i])));
            if (hr > best.v) {
                best.v = hr;
                best.idx = first + i;
            }
        }
    }
    float d[N];
    float m = -3.0e38f;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        d[i] = steer_diff(hp[i], hm[i]);
        m = fmaxf(m, fmaf(hg[i], cf, d[i] * bcf));
    }
    // the estimate is within a few 1e-5 of the exact exponent: half a unit of slack keeps z <= ~0.5
    const int En = max(a.E, exp_ref(m));
    a.s = ldexpf(a.s, a.E - En);
    a.E = En;
    const double nE = -(double)En;
    float t0 = 0.f, t1 = 0.f;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const double dd = (DT == SS_BF16) ? (double)d[i] : steer_diff_d(hp[i], hm[i]);
        const float z = (float)fma((double)hg[i], c, fma(dd, bc, nE));
        if (i & 1) t1 += __builtin_amdgcn_exp2f(z); else t0 += __builtin_amdgcn_exp2f(z);
    }
    a.s += t0 + t1;
}

__device__ __forceinline__ Partial wave_combine(Acc a) {
    const int Em = wave_max_i32(a.E);
    const float S = wave_sum_f32(ldexpf(a.s, a.E - Em));
    return Partial{Em, S};
}

// ------------------------------------------------------------------ row lists

// Which rows a row pass covers: positions [t_lo, t_hi) of every sequence that is still in play.
// The block is verified in at most two such windows (see the host side): Algorithm 1 stops at the
// first rejection, so the later positions of a sequence rejected early never need their rows.
struct RowWindow {
    const int32_t* draft_len;  // NULL => K_b = k_max
    const int32_t* alive;      // NULL => every sequence; else rows only where alive[b] != 0
    int kmax, t_lo, t_hi;
};

// Rows of sequence b inside the window.  A length outside [0, k_max] contributes none
// (the sequence is flagged elsewhere).
__device__ __forceinline__ int window_rows(const RowWindow& w, int b) {
    const int K = w.draft_len ? w.draft_len[b] : w.kmax;
    if (K < 0 || K > w.kmax) return 0;
    if (w.alive && !w.alive[b]) return 0;
    return max(0, min(K, w.t_hi) - w.t_lo);
}

// off[b] = number of window rows before sequence b; off[B] = total.
// Called by every thread of a workgroup of NT threads (NT a multiple of 64, at most 1024);
// `off` may be LDS or global memory.  Ends with a barrier, so `off` is readable on return.
__device__ __forceinline__ void block_scan_rows(const RowWindow& win, int B, int* off, int NT) {
    __shared__ int wave_tot[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, NW = NT >> 6;
    int carry = 0;
    for (int b0 = 0; b0 < B; b0 += NT) {
        const int b = b0 + tid;
        const int k = b < B ? window_rows(win, b) : 0;
        int incl = k;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int y = __shfl_up(incl, d, kWave);
            if (lane >= d) incl += y;
        }
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        int before = carry, all = 0;
        for (int w = 0; w < NW; ++w) {
            const int wt = wave_tot[w];
            if (w < wave) before += wt;
            all += wt;
        }
        if (b < B) off[b] = before + incl - k;
        carry += all;
        __syncthreads();
    }
    if (tid == 0) off[B] = carry;
    __syncthreads();
}

// Only for batches too large for the in-kernel LDS row list.
__global__ __launch_bounds__(1024) void prep_rows_kernel(const RowWindow win, int B, int32_t* __restrict__ row_off) {
    block_scan_rows(win, B, row_off, 1024);
}

// ------------------------------------------------------------------ kernel: row log-sum-exp partials

struct LseArgs {
    const void* G;
    const void* Sm;
    RowWindow win;             // the rows this launch covers
    int uniform_rows;          // > 0: every sequence has exactly this many window rows, no list needed
    int32_t* row_off;          // else: global copy of the row list, [B+1]
    Partial* partial;          // [rows][2][NS]
    long sb, st;               // element strides
    int B, kmax, V, NS;
    int slice_vecs;            // 16-byte vectors per slice
    int list_in_lds;           // build the row list in LDS (else row_off was filled by prep_rows)
    float c_hi;                // fl32(log2(e)/T)
    uint32_t* zero_ptr;        // arrival counters of a split recovery: workgroup 0 clears zero_n of them
    int zero_n;
};

// Work item = (row, tensor, slice), flattened so that consecutive items are consecutive slices
// of one row.  One wave per item, no communication between waves; the grid is persistent and
// strides over the item list.  Ragged batches build the row list in LDS at kernel start
// (every workgroup repeats the same small scan), so no separate launch is needed.
// Workgroup 0 also publishes the row list for the kernels that consume the partials.
template <int DT, int VEC, int kUnroll>
__global__ __launch_bounds__(kLseThreads) void row_lse_kernel(const LseArgs a) {
    extern __shared__ int lds_off[];
    const int lane = threadIdx.x & 63;
    const int wave_global = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * (kLseThreads / kWave) + (threadIdx.x >> 6)));
    const int waves_total = gridDim.x * (kLseThreads / kWave);
    const bool ragged = a.uniform_rows <= 0;
    const int* off = a.row_off;
    if (ragged && a.list_in_lds) {
        block_scan_rows(a.win, a.B, lds_off, kLseThreads);
        off = lds_off;
    }
    if (blockIdx.x == 0 && ragged && a.list_in_lds)
        for (int i = threadIdx.x; i <= a.B; i += kLseThreads) a.row_off[i] = lds_off[i];
    if (blockIdx.x == 0)
        for (int i = threadIdx.x; i < a.zero_n; i += kLseThreads) a.zero_ptr[i] = 0u;
    const int R = ragged ? off[a.B] : a.B * a.uniform_rows;
    const long items = (long)R * 2 * a.NS;
    const long slice_units = a.slice_vecs;
    const long nvec = a.V / VEC;
    const int tailc = a.V - (int)(nvec * VEC);
    constexpr long kGroup = (long)kWave * kUnroll;

    for (long item = wave_global; item < items; item += waves_total) {
        const int k = (int)(item % a.NS);
        const long rx = item / a.NS;
        const int x = (int)(rx & 1);
        const int r = (int)(rx >> 1);
        int b, t;
        if (ragged) {
            int lo = 0, hi = a.B;  // largest b with off[b] <= r; off[B] = R > r
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (off[mid] <= r) lo = mid; else hi = mid;
            }
            b = lo;
            t = a.win.t_lo + (r - off[b]);
        } else {
            b = r / a.uniform_rows;
            t = a.win.t_lo + (r - b * a.uniform_rows);
        }
        const void* row = row_ptr<DT>(x ? a.Sm : a.G, (long)b * a.sb + (long)t * a.st);
        const long v0 = (long)k * slice_units;
        const long v1 = min(nvec, v0 + slice_units);
        const long nfull = v1 > v0 ? (v1 - v0) / kGroup : 0;  // wave-uniform trip count

        Acc acc{kEInit, 0.f};
        long v = v0 + lane;
        for (long g = 0; g < nfull; ++g, v += kGroup) {
            typename RawT<DT, VEC>::type raw[kUnroll];
#pragma unroll
            for (int j = 0; j < kUnroll; ++j) raw[j] = ld_raw<DT, VEC>(row, v + (long)kWave * j);
            float h[kUnroll * VEC];
#pragma unroll
            for (int j = 0; j < kUnroll; ++j) {
                float hj[VEC];
                unpack(raw[j], hj);
#pragma unroll
                for (int i = 0; i < VEC; ++i) h[j * VEC + i] = hj[i];
            }
            acc_add_f32<kUnroll * VEC>(acc, h, a.c_hi);
        }
        for (; v < v1; v += kWave) {
            float hj[VEC];
            unpack(ld_raw<DT, VEC>(row, v), hj);
            acc_add_f32<VEC>(acc, hj, a.c_hi);
        }
        if (k == a.NS - 1 && lane < tailc) {  // logits past the last full vector
            float hj[1] = {ld_elem<DT>(row, nvec * VEC + lane)};
            acc_add_f32<1>(acc, hj, a.c_hi);
        }
        const Partial p = wave_combine(acc);
        if (lane == 0) a.partial[item] = p;
    }
}

// ------------------------------------------------------------------ kernel: accept + recover

struct RecArgs {
    const void* G;
    const void* Sm;          // S_noctx, for the ratio test
    const void* recSp;       // S_ctx and S_noctx as the recovery sweep reads them: both alias G when
    const void* recSm;       //   beta == 0, so that the steering term is an exact zero and costs no HBM traffic
    const int32_t* draft;
    const int32_t* draft_len;
    const float* uniforms;
    // Partials of positions [0, t1) come from the first row pass, those of [t1, k_max) from the
    // second (t1 == k_max when there is only one pass).  off1 / off2 are the passes' row lists;
    // rows1 > 0 means the first pass had that many rows for every sequence and no list.
    const int32_t* off1;
    const int32_t* off2;
    const Partial* partial1;
    const Partial* partial2;
    const int32_t* alive;    // two passes: sequences whose later positions were scored; else NULL
    const int32_t* flagged;  // two passes: bad length or draft id, found by the verdict kernel; else NULL
    const int32_t* first_rej;  // two passes: first rejection inside the first window (verdict kernel)
    int t1, rows1;
    int32_t* accepted_len;
    int32_t* next_token;
    float* next_token_logprob;
    float* recovery_logprobs;
    float* draft_logprobs;
    long sb, st;
    int B, kmax, V;
    int NS, NS2;     // slices per row in the first / second row pass
    int NC;          // chunks per row (full chunks + one pseudo-chunk for the logits past the last vector)
    double c;        // log2(e) / T
    double bc;       // beta * log2(e) / T
    double beta;     // beta itself, for the greedy argmax of Eq. 8
    double ln_lambda;
    double rho;      // (c - fl32(c)) / fl32(c): first-order repair of sums formed with the rounded scale
    float c_hi;      // fl32(c)
    int greedy;      // SS_FLAG_GREEDY
    int plain;       // beta == 0: no steering term, the specialist rows are not read by the recovery sweep
    // Split recovery (small batches): `parts` workgroups share the recovery row of one sequence.
    int parts;
    Partial* chunk_tab;   // [B][NC] chunk masses, filled by the parts
    Best* part_best;      // [B][parts] greedy candidates of the parts
    uint32_t* arrive;     // [B] parts that have delivered; cleared by the first row pass
};

// Hand-over between workgroups that may run on different XCDs, whose L2 caches are not coherent with each
// other, without a cache-wide write-back (a device-scope release fence writes the whole L2 back and costs about
// 40 ns of a serialised resource per fence): the producer writes with device-scope atomic stores, which go
// through to memory, waits for them to complete, and only then bumps the arrival counter; the workgroup that
// sees the counter complete reads with device-scope atomic loads.  Nobody ever waits for anybody.
template <typename T>
__device__ __forceinline__ void st_dev(T* p, T v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
template <typename T>
__device__ __forceinline__ T ld_dev(const T* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_dev_partial(Partial* p, Partial v) {
    st_dev(reinterpret_cast<unsigned long long*>(p),
           ((unsigned long long)__float_as_uint(v.s) << 32) | (unsigned long long)(unsigned)v.E);
}
__device__ __forceinline__ Partial ld_dev_partial(const Partial* p) {
    const unsigned long long w = ld_dev(reinterpret_cast<const unsigned long long*>(p));
    return Partial{(int)(unsigned)(w & 0xFFFFFFFFull), __uint_as_float((unsigned)(w >> 32))};
}
// every memory operation this wave has issued so far has completed: s_waitcnt vmcnt(0) lgkmcnt(0)
__device__ __forceinline__ void wait_stores() { __builtin_amdgcn_s_waitcnt(0x0070); }

// log2 of sum_v 2^(h_v * c) for one row from its slice partials, by one lane: the partials are merged in
// slice order (sixteen loads in flight at a time), so the result does not depend on who computes it.
__device__ __forceinline__ double combine_partials_lane(const Partial* p, int ns, double rho) {
    int Em = kEInit;
    float S = 0.f;
    for (int k0 = 0; k0 < ns; k0 += 16) {
        Partial pv[16];
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (k0 + i < ns) pv[i] = p[k0 + i];
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (k0 + i < ns) {
                const int En = max(Em, pv[i].E);
                S = ldexpf(S, Em - En) + ldexpf(pv[i].s, pv[i].E - En);
                Em = En;
            }
    }
    return (double)Em * (1.0 + rho) + log2((double)S);  // E*rho: see acc_add_f32
}

// PLAIN (beta == 0): the recovery distribution is Softmax(h_LLM / T); the two specialist rows are
// neither loaded nor unpacked, their logits read as 0 so that the steering term is an exact zero.
template <int DT, int VEC, bool PLAIN>
__device__ __forceinline__ void unpack_steer(const typename RawT<DT, VEC>::type& rp, const typename RawT<DT, VEC>::type& rm,
                                             float (&hp)[VEC], float (&hm)[VEC]) {
    if (PLAIN) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) hp[i] = hm[i] = 0.f;
    } else {
        unpack(rp, hp);
        unpack(rm, hm);
    }
}

template <int DT, bool PLAIN>
__device__ __forceinline__ float ld_steer(const void* row, long e) {
    return PLAIN ? 0.f : ld_elem<DT>(row, e);
}

// Probability terms 2^(y - E) of the logits one lane owns in recovery chunk c, laid out so that
// a lane's logits are consecutive in the vocabulary: lane l holds vectors 4l..4l+3 of the chunk.
// The pseudo-chunk c == nch holds the < VEC logits past the last full vector, one per lane.
// cnt[j] says how many entries of p[j] are valid; first[j] is the vocabulary index of p[j][0].
// PLAIN forms the terms as the sweep did, 2^(fma(h, c_hi, -E)) in fp32.
template <int DT, int VEC, bool PLAIN>
__device__ __forceinline__ void chunk_lane_terms(const void* g, const void* sp, const void* sm, long nvec, int tailc,
                                                 long nch, long c, int lane, double cc, double bc, float c_hi, int E,
                                                 float (&p)[kChunkSteps][VEC], long (&first)[kChunkSteps],
                                                 int (&cnt)[kChunkSteps]) {
    const double dE = (double)E;
    const float nE = -(float)E;
    typename RawT<DT, VEC>::type rg[kChunkSteps], rp[kChunkSteps], rm[kChunkSteps];
#pragma unroll
    for (int j = 0; j < kChunkSteps; ++j) {
        const long v = c * (long)(kWave * kChunkSteps) + (long)lane * kChunkSteps + j;
        cnt[j] = 0;
        first[j] = v * VEC;
        if (c < nch && v < nvec) {
            rg[j] = ld_raw<DT, VEC>(g, v);
            if (!PLAIN) {
                rp[j] = ld_raw<DT, VEC>(sp, v);
                rm[j] = ld_raw<DT, VEC>(sm, v);
            }
            cnt[j] = VEC;
        }
    }
#pragma unroll
    for (int j = 0; j < kChunkSteps; ++j) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) p[j][i] = 0.f;
        if (cnt[j]) {
            float hg[VEC], hp[VEC], hm[VEC];
            unpack(rg[j], hg);
            unpack_steer<DT, VEC, PLAIN>(rp[j], rm[j], hp, hm);
#pragma unroll
            for (int i = 0; i < VEC; ++i)
                p[j][i] = PLAIN ? __builtin_amdgcn_exp2f(fmaf(hg[i], c_hi, nE))
                                : __builtin_amdgcn_exp2f((float)(rec_y(hg[i], hp[i], hm[i], cc, bc) - dE));
        }
    }
    if (c >= nch && lane < tailc) {
        first[0] = nvec * VEC + lane;
        cnt[0] = 1;
        const float hg = ld_elem<DT>(g, first[0]);
        p[0][0] = PLAIN ? __builtin_amdgcn_exp2f(fmaf(hg, c_hi, nE))
                        : __builtin_amdgcn_exp2f((float)(rec_y(hg, ld_steer<DT, PLAIN>(sp, first[0]),
                                                               ld_steer<DT, PLAIN>(sm, first[0]), cc, bc) - dE));
    }
}

// (E, s) mass of recovery chunk c, by one wave: sum over the chunk of 2^(y - E).  With a steering term the
// exponent is formed in double (acc_add_rec); PLAIN (beta == 0) has only h_LLM * c to form and takes the
// row pass's route, one fp32 fma per logit with the rounded scale c_hi, repaired to first order by the caller.
template <int DT, int VEC, bool GREEDY, bool PLAIN>
__device__ __forceinline__ Partial chunk_mass(const void* g, const void* sp, const void* sm, long nvec, int tailc,
                                              long nch, long c, int lane, double cc, double bc, double beta,
                                              float c_hi, Best& best) {
    const float cf = (float)cc, bcf = (float)bc;
    Acc acc{kEInit, 0.f};
    if (c < nch) {
        const long vbase = c * (long)(kWave * kChunkSteps) + lane;
        typename RawT<DT, VEC>::type rg[kChunkSteps], rp[kChunkSteps], rm[kChunkSteps];
#pragma unroll
        for (int j = 0; j < kChunkSteps; ++j) {
            const long v = vbase + (long)j * kWave;
            if (v < nvec) {
                rg[j] = ld_raw<DT, VEC>(g, v);
                if (!PLAIN) {
                    rp[j] = ld_raw<DT, VEC>(sp, v);
                    rm[j] = ld_raw<DT, VEC>(sm, v);
                }
            }
        }
        if (PLAIN && vbase + (long)(kChunkSteps - 1) * kWave < nvec) {  // a full chunk: one accumulate over its 4 vectors
            float h[kChunkSteps * VEC];
#pragma unroll
            for (int j = 0; j < kChunkSteps; ++j) {
                float hj[VEC];
                unpack(rg[j], hj);
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    h[j * VEC + i] = hj[i];
                    if (GREEDY && (double)hj[i] > best.v) {
                        best.v = (double)hj[i];
                        best.idx = (vbase + (long)j * kWave) * VEC + i;
                    }
                }
            }
            acc_add_f32<kChunkSteps * VEC>(acc, h, c_hi);
        } else {
#pragma unroll
            for (int j = 0; j < kChunkSteps; ++j) {
                const long v = vbase + (long)j * kWave;
                if (v < nvec) {
                    float hg[VEC], hp[VEC], hm[VEC];
                    unpack(rg[j], hg);
                    unpack_steer<DT, VEC, PLAIN>(rp[j], rm[j], hp, hm);
                    if (PLAIN) {
#pragma unroll
                        for (int i = 0; i < VEC; ++i)
                            if (GREEDY && (double)hg[i] > best.v) {
                                best.v = (double)hg[i];
                                best.idx = v * VEC + i;
                            }
                        acc_add_f32<VEC>(acc, hg, c_hi);
                    } else {
                        acc_add_rec<DT, VEC, GREEDY>(acc, hg, hp, hm, cc, bc, cf, bcf, beta, v * VEC, best);
                    }
                }
            }
        }
    } else if (lane < tailc) {
        const long e = nvec * VEC + lane;
        const float hg[1] = {ld_elem<DT>(g, e)}, hp[1] = {ld_steer<DT, PLAIN>(sp, e)}, hm[1] = {ld_steer<DT, PLAIN>(sm, e)};
        if (PLAIN) {
            if (GREEDY && (double)hg[0] > best.v) {
                best.v = (double)hg[0];
                best.idx = e;
            }
            acc_add_f32<1>(acc, hg, c_hi);
        } else {
            acc_add_rec<DT, 1, GREEDY>(acc, hg, hp, hm, cc, bc, cf, bcf, beta, e, best);
        }
    }
    return wave_combine(acc);
}

// Inverse-CDF draw for one sequence by one wave, from the chunk masses `tab` (LDS) of its
// recovery row: a double-precision scan over the masses finds the chunk holding u*Z, and only
// that chunk is read again to pick the token.  Returns log2 Z; writes the per-sequence outputs.
template <int DT, int VEC, bool GREEDY, bool PLAIN>
__device__ __forceinline__ double sample_wave(const RecArgs& a, int b, int n, int lane, const Partial* tab,
                                              const void* g, const void* sp, const void* sm, long nvec, int tailc,
                                              long nch, Best greedy_pick) {
    const int NC = a.NC;
    const double us = (double)a.uniforms[(long)b * (a.kmax + 1) + a.kmax];
    // each lane owns a contiguous run of `per` chunks
    const int per = (NC + kWave - 1) / kWave;
    const int lo = min(lane * per, NC), hi = min(lo + per, NC);
    int Em = kEInit;
    for (int c = lo; c < hi; ++c) Em = max(Em, tab[c].E);
    const int Estar = wave_max_i32(Em);
    double lsum = 0.0;
    for (int c = lo; c < hi; ++c) lsum += ldexp((double)tab[c].s, tab[c].E - Estar);
    const double incl = wave_incl_scan_f64(lsum);
    const double total = wave_last_f64(incl);
    if (GREEDY) {  // the token is already known; only the normaliser is needed
        const double log2Z = (double)Estar + log2(total) + (PLAIN ? a.rho : 0.0) * (double)Estar;
        const long tok = min(max(greedy_pick.idx, 0l), (long)a.V - 1);
        if (lane == 0) {
            a.accepted_len[b] = n;
            a.next_token[b] = (int32_t)tok;
            if (a.next_token_logprob) a.next_token_logprob[b] = (float)(kLn2 * (greedy_pick.v * a.c - log2Z));
        }
        return log2Z;
    }
    const double excl = wave_shift_up_f64(incl);
    const double target = us * total;

    int cfound = -1, clast = -1;
    double cbase = 0.0, cum = excl;
    for (int c = lo; c < hi; ++c) {
        const double m = ldexp((double)tab[c].s, tab[c].E - Estar);
        if (m > 0.0) clast = c;
        const double cum2 = cum + m;
        if (cfound < 0 && cum2 > target) {
            cfound = c;
            cbase = cum;
        }
        cum = cum2;
    }
    const unsigned long long fmask = __ballot(cfound >= 0);
    int cstar;
    double base;
    bool take_last = false;  // the uniform is not below the total mass (u >= 1 or not a number)
    if (fmask) {
        const int L = first_lane(fmask);
        cstar = __shfl(cfound, L, kWave);
        base = __shfl(cbase, L, kWave);
    } else {
        cstar = max(wave_max_i32(clast), 0);
        base = 0.0;
        take_last = true;
    }

    // re-read that chunk with each lane holding consecutive logits: one scan over the lanes.  The terms are
    // taken relative to the chunk's own exponent reference, 2^(y - Ec), so that the logits that carry the
    // chunk are normal fp32 numbers however far the chunk sits below the row's maximum; `sc` brings them
    // to the scale of the chunk table in double, exactly.
    const int Ec = tab[cstar].E;
    const double dE = (double)Ec;
    const double sc = ldexp(1.0, Ec - Estar);
    // PLAIN sums were formed with the rounded scale c_hi: exponents come back as y_hi = h * c_hi, the true one
    // is y_hi * (1 + rho), and the row's log2-sum moves by rho * E* to first order (see acc_add_f32)
    const double fix = PLAIN ? a.rho : 0.0;
    float p[kChunkSteps][VEC];
    long first[kChunkSteps];
    int cnt[kChunkSteps];
    chunk_lane_terms<DT, VEC, PLAIN>(g, sp, sm, nvec, tailc, nch, cstar, lane, a.c, a.bc, a.c_hi, Ec, p, first, cnt);
    double ls = 0.0;
    long lastpos = -1;
#pragma unroll
    for (int j = 0; j < kChunkSteps; ++j) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            ls += (double)p[j][i] * sc;
            if (i < cnt[j] && p[j][i] > 0.f) lastpos = first[j] + i;
        }
    }
    double cw = wave_shift_up_f64(wave_incl_scan_f64(ls)) + base;
    long mytok = -1;
    float ptok = 0.f, plast = 0.f;
#pragma unroll
    for (int j = 0; j < kChunkSteps; ++j) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            cw += (double)p[j][i] * sc;
            if (i < cnt[j] && p[j][i] > 0.f) plast = p[j][i];
            if (!take_last && mytok < 0 && i < cnt[j] && cw > target) {
                mytok = first[j] + i;
                ptok = p[j][i];
            }
        }
    }
    long tok;
    const unsigned long long hmask = __ballot(mytok >= 0);
    if (hmask) {
        const int L = first_lane(hmask);
        tok = __shfl(mytok, L, kWave);
        ptok = __shfl(ptok, L, kWave);
    } else {
        // rounding between the chunk table and the re-read (or take_last): the last logit of
        // the chunk that still carries probability
        long best = lastpos;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) best = max(best, __shfl_xor(best, d, kWave));
        const unsigned long long omask = __ballot(lastpos == best && best >= 0);
        // the chunk's largest logit is within one unit of Ec, so a positive term always exists unless
        // the row holds something that is not a number; keep the index valid then
        tok = omask ? best : min((long)cstar * (kWave * kChunkSteps * VEC), (long)a.V - 1);
        ptok = omask ? __shfl(plast, first_lane(omask), kWave) : 1.f;
    }
    // the chosen logit's exponent back from its term: 2^(y - Ec) is a normal fp32 number with one
    // ulp of error, so log2 of it is good to ~2e-7 whatever the magnitude of y
    const double ytok_hi = dE + log2((double)ptok);
    const double ytok = ytok_hi + fix * ytok_hi;
    const double log2Z = (double)Estar + log2(total) + fix * (double)Estar;
    if (lane == 0) {
        a.accepted_len[b] = n;
        a.next_token[b] = (int32_t)tok;
        if (a.next_token_logprob) a.next_token_logprob[b] = (float)(kLn2 * (ytok - log2Z));
    }
    return log2Z;
}

// Slice partials of (sequence b, position t, tensor x): from the first row pass for t < t1, from the
// second for t >= t1.
__device__ __forceinline__ const Partial* partials_of(const RecArgs& a, int b, int t, int x) {
    if (t < a.t1) {
        const long r = (a.rows1 > 0 ? (long)b * a.rows1 : (long)a.off1[b]) + t;
        return a.partial1 + (r * 2 + x) * a.NS;
    }
    const long r = (long)a.off2[b] + (t - a.t1);
    return a.partial2 + (r * 2 + x) * a.NS2;
}

// Phase 2 for one sequence by its workgroup of NT threads, on positions [T0, Kt) (those before T0
// are known to have been accepted):
//   2a  every (position, tensor) pair gets a lane: merge the row's slice partials, gather the draft
//       token's logit, leave log P(y_t) in lp[2t + x]        (two memory round trips in all)
//   2b  wave 0: Eq. 7 on every position, first rejection by ballot -> *sh_n (Kt if none)
// A draft id outside the vocabulary among those positions sets *sh_bad.  Ends with a barrier.
template <int DT, int NT>
__device__ __forceinline__ void ratio_test_block(const RecArgs& a, int b, int T0, int Kt, double* lp, int* sh_n,
                                                 int* sh_bad) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kmax = a.kmax, V = a.V;
    for (int q = 2 * T0 + tid; q < 2 * Kt; q += NT) {
        const int t = q >> 1, x = q & 1;
        const int y = a.draft[(long)b * kmax + t];
        const bool ok = (y >= 0 && y < V);
        const long off = (long)b * a.sb + (long)t * a.st;
        const float h = ok ? ld_elem<DT>(row_ptr<DT>(x ? a.Sm : a.G, off), y) : 0.f;
        const double L = combine_partials_lane(partials_of(a, b, t, x), t < a.t1 ? a.NS : a.NS2, a.rho);
        lp[q] = kLn2 * ((double)h * a.c - L);
        if (!ok) *sh_bad = 1;
    }
    __syncthreads();
    if (wave == 0) {
        int first_rej = Kt;
        for (int t0 = T0; t0 < Kt; t0 += kWave) {
            const int t = t0 + lane;
            bool rej = false;
            if (t < Kt) {
                const double alpha = fmin(1.0, exp(lp[2 * t] - lp[2 * t + 1] - a.ln_lambda));  // Eq. 7
                rej = !((double)a.uniforms[(long)b * (kmax + 1) + t] <= alpha);
            }
            const unsigned long long rmask = __ballot(rej);
            if (rmask && first_rej == Kt) first_rej = t0 + first_lane(rmask);
        }
        if (lane == 0) *sh_n = first_rej;
    }
    __syncthreads();
}

// Between the two row passes: the ratio test on the positions of the first window,
// [0, min(K_b, t1)), with exactly the arithmetic of the final kernel.  A sequence rejected there is
// finished as far as verification goes (Algorithm 1 breaks out of the loop at the first
// rejection): its later rows are never scored and its first-rejection index is final.  Every
// draft id of the sequence is range-checked here, so a sequence is flagged exactly as in the
// one-pass schedule.
constexpr int kVerdictThreads = 64;  // one wave per sequence: a lane per (position, tensor) pair is plenty

template <int DT>
__global__ __launch_bounds__(kVerdictThreads) void verdict_kernel(const RecArgs a, int32_t* alive, int32_t* flagged,
                                                              int32_t* first_rej) {
    extern __shared__ double smem_d[];
    __shared__ int sh_n, sh_bad;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int kmax = a.kmax, V = a.V;
    const int K = a.draft_len ? a.draft_len[b] : kmax;
    const bool bad_len = (K < 0 || K > kmax);
    if (tid == 0) {
        sh_bad = bad_len ? 1 : 0;
        sh_n = 0;
    }
    __syncthreads();
    if (!bad_len) {
        bool oob = false;
        for (int t = tid; t < K; t += kVerdictThreads) {
            const int y = a.draft[(long)b * kmax + t];
            oob = oob || y < 0 || y >= V;
        }
        if (oob) sh_bad = 1;
    }
    __syncthreads();
    const int Kt = sh_bad ? 0 : min(K, a.t1);
    ratio_test_block<DT, kVerdictThreads>(a, b, 0, Kt, smem_d, &sh_n, &sh_bad);
    if (tid == 0) {
        const bool bad = sh_bad != 0;
        alive[b] = (!bad && sh_n == Kt && K > a.t1) ? 1 : 0;
        flagged[b] = bad ? 1 : 0;
        first_rej[b] = sh_n;
    }
}

// Best candidate of the wave, left in every lane: larger value, then lower index.
__device__ __forceinline__ void wave_best(Best& best) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const double ov = __shfl_xor(best.v, d, kWave);
        const long oi = __shfl_xor(best.idx, d, kWave);
        if (ov > best.v || (ov == best.v && oi < best.idx)) {
            best.v = ov;
            best.idx = oi;
        }
    }
}

// One workgroup (16 waves) per sequence, everything after the row pass in one launch:
//   2a  every (position, tensor) pair gets a wave: merge its slice partials, gather the draft
//       token's logit, leave log P(y_t) in LDS            (two memory round trips in all)
//   2b  wave 0: Eq. 7 on every position, first rejection by ballot
//   3   all waves stream the three rows at the rejected (or bonus) position once, one (E, s)
//       mass per 2048-logit chunk into LDS
//   4   wave 0 draws the token; optionally all waves sweep the rows again to write log-probs
// Only workgroup barriers separate the steps; nothing crosses workgroups.
//
// SPLIT (small batches, where one workgroup per sequence leaves most of the chip idle): a.parts
// workgroups share a sequence.  Each repeats steps 2a-2b (cheap), takes every a.parts-th group of
// 16 chunks in step 3 and delivers its chunk masses to a table in global memory; the part that
// arrives last (an atomic counter per sequence, no workgroup ever waits for another) runs step 4
// from the complete table.  The deliveries are made and counted by one wave with write-through stores
// (st_dev, wait_stores), and the last part reads them with device-scope loads: no cache-wide fence.
template <int DT, int VEC, bool GREEDY, bool SPLIT, bool PLAIN, int NT>
__global__ __launch_bounds__(NT) void accept_recover_kernel(const RecArgs a) {
    extern __shared__ double smem_d[];
    __shared__ int sh_n, sh_bad, sh_last;
    __shared__ double sh_log2Z;
    __shared__ double sh_best_v[kRecThreads / kWave];  // one slot per wave, or per part in the merge of a split row
    __shared__ long sh_best_i[kRecThreads / kWave];

    const int S = SPLIT ? a.parts : 1;
    const int b = SPLIT ? (int)blockIdx.x / S : (int)blockIdx.x;
    const int part = SPLIT ? (int)blockIdx.x - b * S : 0;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int NW = NT / kWave;
    const int kmax = a.kmax, V = a.V;
    double* lp = smem_d;                                            // [kmax][2] log P_LLM, log P_SLM^-
    Partial* tab = reinterpret_cast<Partial*>(smem_d + 2 * kmax);   // [NC] chunk masses

    const int K = a.draft_len ? a.draft_len[b] : kmax;
    const bool bad_len = (K < 0 || K > kmax) || (a.flagged && a.flagged[b]);
    // Two-pass schedule: a sequence the verdict kernel saw rejected inside the first window keeps
    // that first-rejection index (its later rows were never scored); a sequence still in play after
    // that window is tested here on its remaining positions, any other over all K positions.
    const bool in_play = a.alive && a.alive[b] && !bad_len;
    const bool settled = a.alive && !in_play && !bad_len && K > a.t1;
    const int Kt = bad_len ? 0 : K;
    if (tid == 0) {
        sh_bad = bad_len ? 1 : 0;
        sh_n = settled ? a.first_rej[b] : 0;
    }
    __syncthreads();
    if (!settled) ratio_test_block<DT, NT>(a, b, in_play ? a.t1 : 0, Kt, lp, &sh_n, &sh_bad);
    const bool bad = sh_bad != 0;
    if (a.draft_logprobs && part == 0) {  // valid positions from LDS, padded slots 0, a flagged sequence NaN throughout
        const float nanv = __int_as_float(0x7FC00000);
        for (int i = tid; i < kmax * 2; i += NT)
            a.draft_logprobs[(long)b * kmax * 2 + i] = bad ? nanv : (i < 2 * Kt ? (float)lp[i] : 0.f);
    }
    if (bad) {
        if (tid == 0 && part == 0) {
            a.accepted_len[b] = -1;
            a.next_token[b] = -1;
            if (a.next_token_logprob) a.next_token_logprob[b] = __int_as_float(0x7FC00000);
        }
        return;
    }
    __syncthreads();
    const int n = sh_n;

    // ---- 3
    const long off = (long)b * a.sb + (long)n * a.st;
    const void* g = row_ptr<DT>(a.G, off);
    const void* sp = row_ptr<DT>(a.recSp, off);
    const void* sm = row_ptr<DT>(a.recSm, off);
    const long nvec = V / VEC;
    const int tailc = V - (int)(nvec * VEC);
    const long nch = (nvec + kWave * kChunkSteps - 1) / (kWave * kChunkSteps);
    Best best{-__builtin_huge_val(), 0x7FFFFFFFFFFFFFFFl};
    for (int c = part * NW + wave; c < a.NC; c += NW * S) {
        const Partial p = chunk_mass<DT, VEC, GREEDY, PLAIN>(g, sp, sm, nvec, tailc, nch, c, lane, a.c, a.bc, a.beta, a.c_hi, best);
        if (lane == 0) tab[c] = p;
    }
    if (GREEDY) {
        wave_best(best);
        if (lane == 0) {
            sh_best_v[wave] = best.v;
            sh_best_i[wave] = best.idx;
        }
    }
    __syncthreads();

    if (SPLIT) {  // deliver this part; only the last part to arrive goes on
        if (wave == 0) {
            Partial* gtab = a.chunk_tab + (long)b * a.NC;
            for (int c = lane; c < a.NC; c += kWave)
                if ((c / NW) % S == part) st_dev_partial(gtab + c, tab[c]);
            if (GREEDY) {
                best.v = lane < NW ? sh_best_v[lane] : -__builtin_huge_val();
                best.idx = lane < NW ? sh_best_i[lane] : 0x7FFFFFFFFFFFFFFFl;
                wave_best(best);
                if (lane == 0) {
                    Best* o = a.part_best + (long)b * S + part;
                    st_dev(reinterpret_cast<unsigned long long*>(&o->v), (unsigned long long)__double_as_longlong(best.v));
                    st_dev(reinterpret_cast<unsigned long long*>(&o->idx), (unsigned long long)best.idx);
                }
            }
            wait_stores();  // this wave's deliveries have reached memory before it is counted
            unsigned prev = 0;
            if (lane == 0) prev = __hip_atomic_fetch_add(a.arrive + b, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (lane == 0) sh_last = (prev == (unsigned)(S - 1)) ? 1 : 0;
        }
        __syncthreads();
        if (!sh_last) return;
        if (wave == 0) {
            const Partial* gtab = a.chunk_tab + (long)b * a.NC;
            for (int c = lane; c < a.NC; c += kWave) tab[c] = ld_dev_partial(gtab + c);
            if (GREEDY && lane < S) {
                const Best* o = a.part_best + (long)b * S + lane;
                sh_best_v[lane] = __longlong_as_double((long long)ld_dev(reinterpret_cast<const unsigned long long*>(&o->v)));
                sh_best_i[lane] = (long)ld_dev(reinterpret_cast<const unsigned long long*>(&o->idx));
            }
        }
        __syncthreads();
    }

    // ---- 4
    if (wave == 0) {
        if (GREEDY) {
            const int NB = SPLIT ? S : NW;
            best.v = lane < NB ? sh_best_v[lane] : -__builtin_huge_val();
            best.idx = lane < NB ? sh_best_i[lane] : 0x7FFFFFFFFFFFFFFFl;
            wave_best(best);
        }
        const double log2Z = sample_wave<DT, VEC, GREEDY, PLAIN>(a, b, n, lane, tab, g, sp, sm, nvec, tailc, nch, best);
        if (lane == 0) sh_log2Z = log2Z;
    }
    if (a.recovery_logprobs) {
        __syncthreads();
        const double log2Z = sh_log2Z;
        float* out = a.recovery_logprobs + (long)b * V;
        for (long v = tid; v < nvec; v += NT) {
            float hg[VEC], hp[VEC], hm[VEC];
            unpack(ld_raw<DT, VEC>(g, v), hg);
            if (PLAIN) {
#pragma unroll
                for (int i = 0; i < VEC; ++i) hp[i] = hm[i] = 0.f;
            } else {
                unpack(ld_raw<DT, VEC>(sp, v), hp);
                unpack(ld_raw<DT, VEC>(sm, v), hm);
            }
#pragma unroll
            for (int i = 0; i < VEC; ++i)
                out[v * VEC + i] = (float)(kLn2 * (rec_y(hg[i], hp[i], hm[i], a.c, a.bc) - log2Z));
        }
        if (tid < tailc) {
            const long e = nvec * VEC + tid;
            out[e] = (float)(kLn2 * (rec_y(ld_elem<DT>(g, e), ld_steer<DT, PLAIN>(sp, e), ld_steer<DT, PLAIN>(sm, e), a.c, a.bc) - log2Z));
        }
    }
}

__global__ void zero_u32_kernel(uint32_t* p, int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0u;
}

// ------------------------------------------------------------------ host side

struct Plan {
    int vec;         // logits per 16-byte vector
    int NS, slice_vecs;    // first row pass: slices per row, fast-width vectors per slice
    int NS2, slice_vecs2;  // second row pass
    int NSf, slice_vecsf;  // one pass over all k_max positions (taken when draft_logprobs is requested)
    int t1;          // positions in the first row pass; == k_max when the block is verified in one pass
    size_t off_list2, off_alive, off_flagged, off_firstrej, off_partial;
    size_t off_arrive, off_part_best, off_chunk_tab;  // split recovery; only present for small batches
    size_t bytes;
};

// Small batches split each sequence's recovery row over several workgroups so that the sweep is
// not tied to the rate of one compute unit per sequence: as many parts as there are compute units
// per sequence, but a part is worth having only if it gets a full round of 16 chunks.
constexpr int kSplitMaxBatch = 128;  // workspace is reserved for the split up to this batch (half of MI355X's 256 units)
constexpr int kSplitMaxParts = 16;   // one LDS slot per part in the greedy merge

int recovery_parts(int B, int NC, int cus) {
    if (B < 1 || B > kSplitMaxBatch) return 1;
    const int by_chunks = (NC + (kRecThreads / kWave) - 1) / (kRecThreads / kWave);
    int parts = cus / B;
    if (parts > by_chunks) parts = by_chunks;
    if (parts > kSplitMaxParts) parts = kSplitMaxParts;
    return parts < 1 ? 1 : parts;
}

// Two row passes pay off when the batch is large enough to be bandwidth-bound and long enough for
// a first rejection to cut rows: the first quarter of the positions is scored for everyone, the
// rest only for the sequences that are still in play.
constexpr long kEarlyExitMinBytes = 512l << 20;

int first_window(const ss_params* p) {
    if (p->flags & SS_FLAG_FULL_ROWS) return p->k_max;
    if (p->k_max < 4) return p->k_max;
    const long esz = p->dtype == SS_BF16 ? 2 : 4;
    if ((long)p->batch * p->k_max * 2 * p->vocab * esz < kEarlyExitMinBytes) return p->k_max;
    return p->k_max / 4;
}

bool shape_ok(const ss_params* p) {
    if (!p) return false;
    if (p->batch < 0 || p->k_max < 0 || p->k_max > SS_MAX_K) return false;
    if (p->vocab < 1 || p->vocab > SS_MAX_VOCAB) return false;
    if (p->dtype != SS_F32 && p->dtype != SS_BF16) return false;
    if ((long)p->batch * (p->k_max + 1) > (1l << 30)) return false;
    return true;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int chunks_per_row(int V, int vec) {
    const long nvec = V / vec;
    const long nch = (nvec + kWave * kChunkSteps - 1) / (kWave * kChunkSteps);
    return (int)nch + ((V % vec) ? 1 : 0);
}

// Slices per row for a pass expected to cover `row_tensors` (row, tensor) pairs: 64 KiB slices for
// big passes, smaller ones (down to one unrolled group) when there are too few rows to give every
// resident wave several slices -- a wave that gets one or two long slices cannot balance.
void slice_plan(long nvec, long row_tensors, int& NS, int& slice_vecs) {
    long ns_lo = (nvec + kMaxSliceVecs - 1) / kMaxSliceVecs;
    long ns_hi = (nvec + kMinSliceVecs - 1) / kMinSliceVecs;
    long want = row_tensors > 0 ? (32768 + row_tensors - 1) / row_tensors : 1;
    long ns = want < ns_lo ? ns_lo : (want > ns_hi ? ns_hi : want);
    if (ns > kMaxSlices) ns = kMaxSlices;
    if (ns < 1) ns = 1;
    long sv = (nvec + ns - 1) / ns;
    sv = (sv + kMinSliceVecs - 1) / kMinSliceVecs * kMinSliceVecs;
    ns = (nvec + sv - 1) / sv;
    if (ns < 1) ns = 1;
    NS = (int)ns;
    slice_vecs = (int)sv;
}

Plan make_plan(const ss_params* p) {
    Plan pl;
    pl.vec = p->dtype == SS_BF16 ? 8 : 4;
    const long nvec = (p->vocab + pl.vec - 1) / pl.vec;
    pl.t1 = first_window(p);
    const long rows1 = (long)p->batch * pl.t1, rows2 = (long)p->batch * (p->k_max - pl.t1);
    slice_plan(nvec, rows1 * 2, pl.NS, pl.slice_vecs);
    // the second pass covers only the sequences still in play: typically a third of the padded rows
    slice_plan(nvec, rows2 * 2 / 3, pl.NS2, pl.slice_vecs2);
    slice_plan(nvec, (long)p->batch * p->k_max * 2, pl.NSf, pl.slice_vecsf);
    const size_t B = (size_t)p->batch;
    size_t o = align_up((B + 1) * sizeof(int32_t), 256);  // row list of the first pass
    pl.off_list2 = o;    o += align_up((B + 1) * sizeof(int32_t), 256);      // row list of the second pass
    pl.off_alive = o;    o += align_up((B ? B : 1) * sizeof(int32_t), 256);
    pl.off_flagged = o;  o += align_up((B ? B : 1) * sizeof(int32_t), 256);
    pl.off_firstrej = o; o += align_up((B ? B : 1) * sizeof(int32_t), 256);
    pl.off_partial = o;
    // sized for the one-pass schedule as well (a call that asks for draft_logprobs takes it): all
    // k_max positions at the finer of the two slicings
    size_t ns_max = (size_t)(pl.NS > pl.NS2 ? pl.NS : pl.NS2);
    if ((size_t)pl.NSf > ns_max) ns_max = (size_t)pl.NSf;
    o += align_up(((size_t)p->batch * p->k_max * 2 + 1) * ns_max * sizeof(Partial), 256);
    pl.off_arrive = pl.off_part_best = pl.off_chunk_tab = o;
    if (p->batch >= 1 && p->batch <= kSplitMaxBatch) {
        pl.off_arrive = o;     o += align_up(B * sizeof(uint32_t), 256);
        pl.off_part_best = o;  o += align_up(B * kSplitMaxParts * sizeof(Best), 256);
        pl.off_chunk_tab = o;  o += align_up(B * (size_t)chunks_per_row(p->vocab, pl.vec) * sizeof(Partial), 256);
    }
    pl.bytes = o;
    return pl;
}

// One row pass over window `win`.  `uniform_rows` > 0 when every sequence has that many rows.
template <int DT, int VEC>
void launch_row_pass(LseArgs la, const RowWindow& win, int uniform_rows, int32_t* row_off, Partial* partial,
                     long max_rows, hipStream_t stream) {
    const int B = la.B;
    const int cus = device_cu_count();
    la.win = win;
    la.uniform_rows = uniform_rows;
    la.row_off = row_off;
    la.partial = partial;
    const bool listed = uniform_rows <= 0;
    // the row list is built in LDS by the row pass unless the batch is too large for it
    const bool global_list = listed && B > kMaxLdsBatch;
    la.list_in_lds = (listed && !global_list) ? 1 : 0;
    if (global_list) hipLaunchKernelGGL(prep_rows_kernel, dim3(1), dim3(1024), 0, stream, win, B, row_off);
    const long items = max_rows * 2 * la.NS;
    if (items <= 0) return;
    const long per_wg = kLseThreads / kWave;
    long wgs = (items + per_wg - 1) / per_wg;
    const long cap = (long)cus * kLseWgPerCu;
    if (wgs > cap) wgs = cap;
    const size_t lds = la.list_in_lds ? (size_t)(B + 1) * sizeof(int) : 0;
    hipLaunchKernelGGL((row_lse_kernel<DT, VEC, kLseUnroll>), dim3((unsigned)wgs), dim3(kLseThreads), lds,
                       stream, la);
}

template <int DT, int VEC>
hipError_t launch_all(LseArgs la, RecArgs ra, const Plan& pl, char* ws, hipStream_t stream, hipEvent_t* ev) {
    const int B = ra.B, kmax = ra.kmax, V = ra.V;
    int32_t* off1 = reinterpret_cast<int32_t*>(ws);
    int32_t* off2 = reinterpret_cast<int32_t*>(ws + pl.off_list2);
    int32_t* alive = reinterpret_cast<int32_t*>(ws + pl.off_alive);
    int32_t* flagged = reinterpret_cast<int32_t*>(ws + pl.off_flagged);
    int32_t* first_rej = reinterpret_cast<int32_t*>(ws + pl.off_firstrej);
    Partial* partial1 = reinterpret_cast<Partial*>(ws + pl.off_partial);
    // the verdict's position-by-position log-probs are only complete in the one-pass schedule
    const int t1 = ra.draft_logprobs ? kmax : pl.t1;
    const bool two_pass = t1 < kmax;
    hipError_t ev_err = hipSuccess;
    auto mark = [&](int i) {  // stage boundary of the timed entry point
        if (!ev) return;
        const hipError_t e = hipEventRecord(ev[i], stream);
        if (e != hipSuccess && ev_err == hipSuccess) ev_err = e;
    };
    if (t1 != pl.t1) {  // one pass although the plan was made for two
        la.NS = pl.NSf;
        la.slice_vecs = pl.slice_vecsf;
    }
    Partial* partial2 = partial1 + (size_t)B * t1 * 2 * la.NS;
    ra.NS = la.NS;
    ra.NS2 = pl.NS2;
    const bool ragged = ra.draft_len != nullptr && kmax > 0;

    ra.t1 = t1;
    ra.rows1 = ragged ? 0 : t1;
    ra.off1 = off1; ra.off2 = off2; ra.partial1 = partial1; ra.partial2 = partial2;
    ra.alive = two_pass ? alive : nullptr;
    ra.flagged = two_pass ? flagged : nullptr;
    ra.first_rej = two_pass ? first_rej : nullptr;
    ra.NC = chunks_per_row(V, VEC);
    const int cus = device_cu_count();
    ra.parts = recovery_parts(B, ra.NC, cus);
    ra.arrive = reinterpret_cast<uint32_t*>(ws + pl.off_arrive);
    ra.part_best = reinterpret_cast<Best*>(ws + pl.off_part_best);
    ra.chunk_tab = reinterpret_cast<Partial*>(ws + pl.off_chunk_tab);
    const bool split = ra.parts > 1;
    la.zero_ptr = ra.arrive;
    la.zero_n = split ? B : 0;
    const size_t smem = (size_t)2 * kmax * sizeof(double) + (size_t)ra.NC * sizeof(Partial);

    mark(0);
    if (kmax == 0 && split)  // no row pass to clear the arrival counters
        hipLaunchKernelGGL(zero_u32_kernel, dim3(1), dim3(kSplitMaxBatch), 0, stream, ra.arrive, B);
    if (kmax > 0)
        launch_row_pass<DT, VEC>(la, RowWindow{ragged ? ra.draft_len : nullptr, nullptr, kmax, 0, t1},
                                          ragged ? 0 : t1, off1, partial1, (long)B * t1, stream);
    mark(1);
    if (two_pass)
        hipLaunchKernelGGL((verdict_kernel<DT>), dim3((unsigned)B), dim3(kVerdictThreads), (size_t)2 * kmax * sizeof(double),
                           stream, ra, alive, flagged, first_rej);
    mark(2);
    if (two_pass) {
        la.NS = pl.NS2;
        la.slice_vecs = pl.slice_vecs2;
        la.zero_n = 0;
        launch_row_pass<DT, VEC>(la, RowWindow{ra.draft_len, alive, kmax, t1, kmax}, 0, off2, partial2,
                                          (long)B * (kmax - t1), stream);
    }
    mark(3);
    // accept + recover: LDS holds the per-position log-probs and one mass per recovery chunk
    const dim3 rec_grid((unsigned)(B * ra.parts));
    using RecKernel = void (*)(RecArgs);
    constexpr int kFull = kRecThreads, kHalf = kRecThreadsHalf;
    static const RecKernel rec_kernels[8] = {  // index: greedy | split << 1 | plain << 2
        accept_recover_kernel<DT, VEC, false, false, false, kFull>, accept_recover_kernel<DT, VEC, true, false, false, kFull>,
        accept_recover_kernel<DT, VEC, false, true, false, kFull>,  accept_recover_kernel<DT, VEC, true, true, false, kFull>,
        accept_recover_kernel<DT, VEC, false, false, true, kFull>,  accept_recover_kernel<DT, VEC, true, false, true, kFull>,
        accept_recover_kernel<DT, VEC, false, true, true, kFull>,   accept_recover_kernel<DT, VEC, true, true, true, kFull>};
    // With at least two sequences per compute unit, two 8-wave workgroups share a unit: the serial ends of one
    // sequence (ratio test, token pick) then overlap the sweep of another.  Same waves per unit, same arithmetic.
    static const RecKernel rec_kernels_half[4] = {  // index: greedy | plain << 1
        accept_recover_kernel<DT, VEC, false, false, false, kHalf>, accept_recover_kernel<DT, VEC, true, false, false, kHalf>,
        accept_recover_kernel<DT, VEC, false, false, true, kHalf>,  accept_recover_kernel<DT, VEC, true, false, true, kHalf>};
    if (!split && B >= 2 * cus)
        hipLaunchKernelGGL(rec_kernels_half[(ra.greedy ? 1 : 0) | (ra.plain ? 2 : 0)], rec_grid, dim3(kHalf), smem,
                           stream, ra);
    else
        hipLaunchKernelGGL(rec_kernels[(ra.greedy ? 1 : 0) | (split ? 2 : 0) | (ra.plain ? 4 : 0)], rec_grid,
                           dim3(kFull), smem, stream, ra);
    mark(4);
    const hipError_t launch_err = hipGetLastError();
    return launch_err != hipSuccess ? launch_err : ev_err;
}

ss_status verify_block_impl(const void* G, const void* S_ctx, const void* S_noctx, const int32_t* draft,
                            const int32_t* draft_len, const float* uniforms, const ss_params* params,
                            int32_t* accepted_len, int32_t* next_token, float* next_token_logprob,
                            float* recovery_logprobs, float* draft_logprobs, void* workspace,
                            size_t workspace_bytes, void* stream, hipEvent_t* ev) {
    if (!params) return SS_ERR_NULL;
    if (params->dtype != SS_F32 && params->dtype != SS_BF16) return SS_ERR_DTYPE;
    if (!shape_ok(params)) return SS_ERR_SHAPE;
    if (!G || !S_ctx || !S_noctx || !uniforms || !accepted_len || !next_token) return SS_ERR_NULL;
    if (params->k_max > 0 && !draft) return SS_ERR_NULL;
    if (!(params->lambda > 0.f) || !std::isfinite(params->lambda)) return SS_ERR_PARAM;
    if (!(params->temperature > 0.f) || !std::isfinite(params->temperature)) return SS_ERR_PARAM;
    if (!std::isfinite(params->beta)) return SS_ERR_PARAM;
    if ((params->flags & ~(uint32_t)(SS_FLAG_GREEDY | SS_FLAG_FULL_ROWS)) != 0) return SS_ERR_PARAM;
    const long V = params->vocab;
    if (params->stride_t < 0 || params->stride_b < 0) return SS_ERR_STRIDE;
    const long st = params->stride_t ? params->stride_t : V;
    const long sb = params->stride_b ? params->stride_b : (long)(params->k_max + 1) * st;
    if (st < V || sb < (long)params->k_max * st + V) return SS_ERR_STRIDE;
    // logits must sit on element boundaries; the 16-byte loads themselves need no more than that
    const uintptr_t esz = params->dtype == SS_BF16 ? 2 : 4;
    if (((reinterpret_cast<uintptr_t>(G) | reinterpret_cast<uintptr_t>(S_ctx) | reinterpret_cast<uintptr_t>(S_noctx)) &
         (esz - 1)) != 0)
        return SS_ERR_STRIDE;
    const Plan pl = make_plan(params);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0 || workspace_bytes < pl.bytes)
        return SS_ERR_WORKSPACE;
    if (params->batch == 0) return SS_OK;


    char* ws = static_cast<char*>(workspace);

    const double T = (double)params->temperature;
    const double c = kLog2e / T;
    const float c_hi = (float)c;  // the row pass scales by this; the merge repairs the difference

    LseArgs la;
    la.G = G; la.Sm = S_noctx; la.row_off = nullptr; la.partial = nullptr; la.uniform_rows = 0;
    la.win = RowWindow{nullptr, nullptr, params->k_max, 0, params->k_max};
    la.sb = sb; la.st = st; la.B = params->batch; la.kmax = params->k_max; la.V = params->vocab;
    la.NS = pl.NS; la.slice_vecs = pl.slice_vecs; la.list_in_lds = 0; la.c_hi = c_hi;
    la.zero_ptr = nullptr; la.zero_n = 0;

    RecArgs ra;
    const bool steer = params->beta != 0.f;
    ra.G = G; ra.Sm = S_noctx; ra.recSp = steer ? S_ctx : G; ra.recSm = steer ? S_noctx : G; ra.draft = draft; ra.draft_len = draft_len; ra.uniforms = uniforms;
    ra.accepted_len = accepted_len; ra.next_token = next_token;
    ra.next_token_logprob = next_token_logprob; ra.recovery_logprobs = recovery_logprobs;
    ra.draft_logprobs = draft_logprobs; ra.sb = sb; ra.st = st; ra.B = params->batch; ra.kmax = params->k_max;
    ra.V = params->vocab; ra.NS = pl.NS; ra.NS2 = pl.NS2; ra.NC = 0; ra.c = c;
    ra.bc = (double)params->beta * c; ra.ln_lambda = std::log((double)params->lambda);
    ra.rho = (c - (double)c_hi) / (double)c_hi;
    ra.beta = (double)params->beta;
    ra.greedy = (params->flags & SS_FLAG_GREEDY) ? 1 : 0;
    ra.plain = steer ? 0 : 1;
    ra.c_hi = c_hi;
    ra.parts = 1; ra.chunk_tab = nullptr; ra.part_best = nullptr; ra.arrive = nullptr;

    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t err;
    if (params->dtype == SS_BF16) {
        err = launch_all<SS_BF16, 8>(la, ra, pl, ws, s, ev);
    } else {
        err = launch_all<SS_F32, 4>(la, ra, pl, ws, s, ev);
    }
    return err == hipSuccess ? SS_OK : SS_ERR_DEVICE;
}

// ------------------------------------------------------------------ library-owned scratch for callers that cannot allocate

// specsteer_verify_block_static runs the block with this array as its workspace.  Every GPU the library runs
// on holds its own copy until the process ends.  In host code the array's name is only a handle for the lookup
// below, never an address to hand to a kernel: the device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[SS_STATIC_SCRATCH_BYTES];

// Device address of `scratch` on the current device (looked up with that device current, on the first call
// there); NULL if the lookup fails.  Host threads may race to fill an entry, all with the same value.
void* static_scratch_ptr() {
    static std::atomic<void*> ptrs[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    void* p = ptrs[dev].load(std::memory_order_acquire);
    if (!p) {
        void* q = nullptr;
        if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) return nullptr;
        ptrs[dev].store(q, std::memory_order_release);
        p = q;
    }
    return p;
}

}  // namespace

extern "C" {

size_t specsteer_workspace_bytes(const ss_params* params) {
    if (!shape_ok(params)) return 0;
    return make_plan(params).bytes;
}

ss_status specsteer_verify_block(const void* G, const void* S_ctx, const void* S_noctx, const int32_t* draft,
                                 const int32_t* draft_len, const float* uniforms, const ss_params* params,
                                 int32_t* accepted_len, int32_t* next_token, float* next_token_logprob,
                                 float* recovery_logprobs, float* draft_logprobs, void* workspace,
                                 size_t workspace_bytes, void* stream) {
    return verify_block_impl(G, S_ctx, S_noctx, draft, draft_len, uniforms, params, accepted_len, next_token,
                             next_token_logprob, recovery_logprobs, draft_logprobs, workspace, workspace_bytes,
                             stream, nullptr);
}

ss_status specsteer_verify_block_timed(const void* G, const void* S_ctx, const void* S_noctx, const int32_t* draft,
                                       const int32_t* draft_len, const float* uniforms, const ss_params* params,
                                       int32_t* accepted_len, int32_t* next_token, float* next_token_logprob,
                                       float* recovery_logprobs, float* draft_logprobs, void* workspace,
                                       size_t workspace_bytes, void* stream, float* stage_ms) {
    if (!stage_ms) return SS_ERR_NULL;
    for (int i = 0; i < SS_NUM_STAGES; ++i) stage_ms[i] = 0.f;
    hipEvent_t ev[SS_NUM_STAGES + 1];
    int made = 0;
    for (; made <= SS_NUM_STAGES; ++made)
        if (hipEventCreate(&ev[made]) != hipSuccess) break;
    ss_status st = SS_ERR_DEVICE;
    if (made == SS_NUM_STAGES + 1) {
        st = verify_block_impl(G, S_ctx, S_noctx, draft, draft_len, uniforms, params, accepted_len, next_token,
                               next_token_logprob, recovery_logprobs, draft_logprobs, workspace, workspace_bytes,
                               stream, ev);
        if (st == SS_OK && params->batch > 0) {
            if (hipEventSynchronize(ev[SS_NUM_STAGES]) != hipSuccess) st = SS_ERR_DEVICE;
            for (int i = 0; st == SS_OK && i < SS_NUM_STAGES; ++i)
                if (hipEventElapsedTime(&stage_ms[i], ev[i], ev[i + 1]) != hipSuccess) st = SS_ERR_DEVICE;
        }
    }
    for (int i = 0; i < made; ++i) (void)hipEventDestroy(ev[i]);
    return st;
}

ss_status specsteer_verify_block_static(const void* G, const void* S_ctx, const void* S_noctx, const int32_t* draft,
                                        const int32_t* draft_len, const float* uniforms, const ss_params* params,
                                        int32_t* accepted_len, int32_t* next_token, float* next_token_logprob,
                                        float* recovery_logprobs, float* draft_logprobs, void* stream) {
    if (!params) return SS_ERR_NULL;
    if (params->dtype != SS_F32 && params->dtype != SS_BF16) return SS_ERR_DTYPE;
    if (!shape_ok(params)) return SS_ERR_SHAPE;
    if (make_plan(params).bytes > (size_t)SS_STATIC_SCRATCH_BYTES) return SS_ERR_WORKSPACE;  // block too large for the static scratch
    void* ws = static_scratch_ptr();
    if (!ws) return SS_ERR_DEVICE;
    return verify_block_impl(G, S_ctx, S_noctx, draft, draft_len, uniforms, params, accepted_len, next_token,
                             next_token_logprob, recovery_logprobs, draft_logprobs, ws, (size_t)SS_STATIC_SCRATCH_BYTES,
                             stream, nullptr);
}

int specsteer_first_window(const ss_params* params) {
    if (!shape_ok(params)) return -1;
    return first_window(params);
}

const char* specsteer_status_string(int status) {
    switch (status) {
        case SS_OK: return "ok";
        case SS_ERR_NULL: return "a required pointer is NULL";
        case SS_ERR_SHAPE: return "batch, k_max or vocab out of range";
        case SS_ERR_DTYPE: return "unknown logits dtype";
        case SS_ERR_PARAM: return "lambda, beta, temperature or flags out of range";
        case SS_ERR_STRIDE: return "strides negative or rows overlap";
        case SS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case SS_ERR_DEVICE: return "HIP launch failed";
        default: return "unknown status";
    }
}

int specsteer_version(void) { return 100; }

}  // extern "C"
