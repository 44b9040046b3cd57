// Deployment split of SpecSteer's recovery step for MI355X (gfx950).
//
// The paper's deployment appendix (its downlink step) does not ship full-vocabulary logits from
// the cloud to the edge on a rejection: the cloud forms the non-private part of Eq. 8,
//     h_cloud = h_LLM - beta * h_SLM^-,
// keeps its top-k entries (k = 32), and the edge adds beta * h_SLM^+ on those entries and
// resamples.  The two kernels here are those two halves; what they compute, the order of the
// payload and the handling of ties are stated in include/specsteer.h.
//
//   cloud_topk    one 16-wave workgroup per sequence streams the two rows once, screening in fp32
//                 and remembering only per-lane group maxima; those give a lower bound on the
//                 k-th largest logit without any cross-lane work in the stream, and only the few
//                 vectors that reach the bound are read again and evaluated exactly in double.
//                 The survivors (100-200 of 128 K) are ranked by the 16 waves together.  A row degenerate enough
//                 to overflow the survivor buffer falls back to an exact insertion-based path.
//   edge_resample one wave per sequence: lane j owns payload entry j, gathers h_SLM^+ at its
//                 token, and the softmax over the k candidates, the inverse-CDF scan and the
//                 pick are a handful of cross-lane operations in double.
//
// h_cloud is evaluated as one rounded product and one rounded difference in double (no fused
// multiply-add), so the selected set and its order are reproducible bit for bit.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "device_common.h"
#include "specsteer.h"

namespace {

constexpr int kTopThreads = 1024;
constexpr int kTopWaves = kTopThreads / kWave;
constexpr int kTopUnroll = 2;  // vectors per tensor in flight per lane
constexpr int kEdgeThreads = 256;

// The non-private part of Eq. 8, h_LLM - beta * h_SLM^-, exactly rounded step by step.  A token the
// generalist masks (-inf) stays at -inf whatever the specialist says (not -inf + inf).
__device__ __forceinline__ double cloud_logit(float hg, float hm, double beta) {
    return hg == -__builtin_huge_valf() ? -__builtin_huge_val() : __dsub_rn((double)hg, __dmul_rn(beta, (double)hm));
}

// total order of the payload: larger value first, then smaller token id
__device__ __forceinline__ bool beats(double av, int ai, double bv, int bi) {
    return av > bv || (av == bv && ai < bi);
}

__device__ __forceinline__ double readlane_f64(double x, int lane) {
    const long long b = __double_as_longlong(x);
    const int lo = __builtin_amdgcn_readlane((int)(b & 0xFFFFFFFFll), lane);
    const int hi = __builtin_amdgcn_readlane((int)(b >> 32), lane);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

struct TopArgs {
    const void* G;
    const void* Sm;
    const int32_t* row;
    int32_t* out_index;
    float* out_value;
    long sb, st;
    int B, kmax, V, topk;
    double beta;
};

// A wave's running best list: lane j holds the j-th best entry seen so far (all 64 lanes are
// kept sorted; only the first topk matter).  tau is the entry at lane topk-1.
struct WaveTop {
    double ev;
    int ei;
    double tau_v;
    int tau_i;
};

__device__ __forceinline__ void wave_insert(WaveTop& w, double cv, int ci, int lane, int topk) {
    if (!beats(cv, ci, w.tau_v, w.tau_i)) return;  // wave-uniform
    const unsigned long long ahead = __ballot(beats(w.ev, w.ei, cv, ci));  // a prefix of the lanes
    const int pos = __popcll(ahead);
    const double sv = wave_shift_up_f64(w.ev);
    const int si = __builtin_amdgcn_update_dpp(0, w.ei, kDppWaveShr1, 0xF, 0xF, false);
    if (lane > pos) {
        w.ev = sv;
        w.ei = si;
    } else if (lane == pos) {
        w.ev = cv;
        w.ei = ci;
    }
    w.tau_v = readlane_f64(w.ev, topk - 1);
    w.tau_i = __builtin_amdgcn_readlane(w.ei, topk - 1);
}

__device__ __forceinline__ double permute_f64(double x, int dst_lane) {
    const long long b = __double_as_longlong(x);
    const int lo = __builtin_amdgcn_ds_permute(dst_lane << 2, (int)(b & 0xFFFFFFFFll));
    const int hi = __builtin_amdgcn_ds_permute(dst_lane << 2, (int)(b >> 32));
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

// Offer every lane's candidate (hc, idx) flagged in mask m to the wave's list, lowest lane first.
__device__ __forceinline__ void wave_offer(WaveTop& w, unsigned long long m, double hc, int idx, int lane, int topk) {
    while (m) {
        const int L = first_lane(m);
        m &= m - 1;
        wave_insert(w, readlane_f64(hc, L), __builtin_amdgcn_readlane(idx, L), lane, topk);
    }
}

// Exact but slow path, taken only when the candidate buffer of the fast path overflows (rows with
// thousands of equal top values): every wave keeps its own best-k list sorted across its lanes and
// inserts newcomers one at a time; the 16 lists are merged by rank in LDS (c_v, c_i: 1024 entries).
template <int DT, int VEC>
__device__ void topk_by_insertion(const TopArgs& a, const void* g, const void* sm, int32_t* oi, float* ov, double* c_v,
                                  int* c_i) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int topk = a.topk, V = a.V;
    const long nvec = V / VEC;
    const int tailc = V - (int)(nvec * VEC);
    const double ninf = -__builtin_huge_val();

    // An empty slot is (-inf, id >= V); the ids differ per lane so that the order stays total.
    WaveTop w{ninf, 0x7FFFFFFF - lane, ninf, 0x7FFFFFFF};
    bool seeded = false;
    constexpr long kStep = (long)kTopWaves * kWave;  // vectors the workgroup covers per step
    for (long v0 = (long)wave * kWave; v0 < nvec; v0 += kStep * kTopUnroll) {
        typename RawT<DT, VEC>::type rg[kTopUnroll], rm[kTopUnroll];
        bool valid[kTopUnroll];
#pragma unroll
        for (int j = 0; j < kTopUnroll; ++j) {
            const long v = v0 + j * kStep + lane;
            valid[j] = v < nvec;
            if (valid[j]) {
                rg[j] = ld_raw<DT, VEC>(g, v);
                rm[j] = ld_raw<DT, VEC>(sm, v);
            }
        }
#pragma unroll
        for (int j = 0; j < kTopUnroll; ++j) {
            if (v0 + j * kStep >= nvec) break;  // wave-uniform
            float hg[VEC], hm[VEC];
            if (valid[j]) {
                unpack(rg[j], hg);
                unpack(rm[j], hm);
            }
            double hc[VEC];
            bool mine = false;
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                hc[i] = valid[j] ? cloud_logit(hg[i], hm[i], a.beta) : ninf;
                mine = mine || (valid[j] && hc[i] >= w.tau_v);  // cheap screen; the exact order is applied below
            }
            const int idx0 = (int)((v0 + j * kStep + lane) * VEC);
            int ifirst = 0;
            if (!seeded) {
                // Seed the list with one logit per lane, sorted by counting, instead of 64 insertions:
                // each lane counts the lanes whose entry precedes its own and sends its entry there.
                seeded = true;
                ifirst = 1;
                const double sv = hc[0];
                const int si = valid[j] ? idx0 : 0x7FFFFFFF - lane;
                int rank = 0;
                for (int L = 0; L < kWave; ++L)
                    rank += beats(readlane_f64(sv, L), __builtin_amdgcn_readlane(si, L), sv, si) ? 1 : 0;
                w.ev = permute_f64(sv, rank);
                w.ei = __builtin_amdgcn_ds_permute(rank << 2, si);
                w.tau_v = readlane_f64(w.ev, topk - 1);
                w.tau_i = __builtin_amdgcn_readlane(w.ei, topk - 1);
                mine = true;
            }
            if (__ballot(mine) == 0ull) continue;  // nothing in this vector reaches the list: the common case
#pragma unroll
            for (int i = 0; i < VEC; ++i) {
                if (i < ifirst) continue;
                const int idx = idx0 + i;
                wave_offer(w, __ballot(valid[j] && beats(hc[i], idx, w.tau_v, w.tau_i)), hc[i], idx, lane, topk);
            }
        }
    }
    if (tailc && wave == 0) {  // logits past the last full vector
        const bool valid = lane < tailc;
        const int e = (int)(nvec * VEC) + lane;
        const double hc = valid ? cloud_logit(ld_elem<DT>(g, e), ld_elem<DT>(sm, e), a.beta)
                                : ninf;
        wave_offer(w, __ballot(valid && beats(hc, e, w.tau_v, w.tau_i)), hc, e, lane, topk);
    }

    // The 16 sorted lists meet in LDS.  A candidate's rank in the merged order is its own
    // position plus, for every other list, the number of entries that precede it there
    // (a binary search, the lists being sorted); ranks are unique because token ids are.
    c_v[wave * kWave + lane] = w.ev;
    c_i[wave * kWave + lane] = w.ei;
    __syncthreads();
    if (lane < topk && w.ei < V) {
        int rank = lane;
        for (int u = 0; u < kTopWaves; ++u) {
            if (u == wave) continue;
            int lo = 0, hi = topk;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (beats(c_v[u * kWave + mid], c_i[u * kWave + mid], w.ev, w.ei)) lo = mid + 1; else hi = mid;
            }
            rank += lo;
        }
        if (rank < topk) {
            oi[rank] = w.ei;
            ov[rank] = (float)w.ev;
        }
    }
}

// Fast path, one HBM pass.  No lane talks to another while the rows stream:
//   A  each lane screens its logits in fp32 (h = fma(-beta, h_SLM^-, h_LLM): correctly rounded, so
//      within 2^-24 of the double value) and keeps only the maximum of each group of its vectors
//      (kTopSlots groups per lane, in LDS) and its overall maximum;
//   B  a lane's maximum, lowered by the rounding margin, is a lower bound on a real logit of
//      that lane, and different lanes own different logits: the minimum over the 16 waves of each
//      wave's r-th largest bound, r = ceil(k/16), has at least k logits at or above it, so it is
//      a lower bound tau on the k-th largest logit of the row;
//   C  only the vector groups whose recorded maximum reaches tau are read again (a few dozen
//      vectors per row); their logits are evaluated exactly in double and those >= tau go to a
//      candidate buffer in LDS (typically 100-200 entries);
//   D  each candidate counts the candidates that precede it in the payload order; ranks below k
//      write themselves to the payload.
constexpr int kTopSlots = 16;  // one vector per group up to 16 K vectors per row
constexpr int kTopCap = 1024;  // candidate buffer entries; more means a degenerate row -> exact slow path
constexpr int kTopTodo = 2048; // (lane, group) pairs queued for the exact re-read

__device__ __forceinline__ float wave_max_f32(float x) {
    x = fmaxf(x, __int_as_float(dpp_mov<kDppXor1>(__float_as_int(x))));
    x = fmaxf(x, __int_as_float(dpp_mov<kDppXor2>(__float_as_int(x))));
    x = fmaxf(x, __int_as_float(dpp_mov<kDppHalfMirror>(__float_as_int(x))));
    x = fmaxf(x, __int_as_float(dpp_mov<kDppMirror>(__float_as_int(x))));
    const int v = __float_as_int(x);
    const float a = __int_as_float(__builtin_amdgcn_readlane(v, 0)), b = __int_as_float(__builtin_amdgcn_readlane(v, 16));
    const float c = __int_as_float(__builtin_amdgcn_readlane(v, 32)), d = __int_as_float(__builtin_amdgcn_readlane(v, 48));
    return fmaxf(fmaxf(a, b), fmaxf(c, d));
}

template <int DT, int VEC>
__global__ __launch_bounds__(kTopThreads) void cloud_topk_kernel(const TopArgs a) {
    __shared__ float gm[kTopSlots * kTopThreads];  // group maxima, [slot][thread]
    __shared__ double c_v[kTopCap];
    __shared__ int c_i[kTopCap];
    __shared__ float wave_bound[kTopWaves];
    __shared__ int todo[kTopTodo];
    __shared__ int cand_count, todo_count;
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int topk = a.topk, V = a.V;
    int32_t* oi = a.out_index + (long)b * topk;
    float* ov = a.out_value + (long)b * topk;
    if (tid < topk) {  // slots that no candidate claims (V < k, or a flagged sequence)
        oi[tid] = -1;
        ov[tid] = -__builtin_huge_valf();
    }
    if (tid == 0) {
        cand_count = 0;
        todo_count = 0;
    }
    const int r = a.row[b];
    if (r < 0 || r > a.kmax) return;
    const long off = (long)b * a.sb + (long)r * a.st;
    const void* g = row_ptr<DT>(a.G, off);
    const void* sm = row_ptr<DT>(a.Sm, off);
    const long nvec = V / VEC;
    const int tailc = V - (int)(nvec * VEC);
    const float nbeta = -(float)a.beta;  // beta arrives as an fp32 value, so this is exact
    const float ninf = -__builtin_huge_valf();

    // ---- A: stream; vector q of this lane is q * 1024 + tid
    const int Q = (int)((nvec + kTopThreads - 1) / kTopThreads);
    const int gsz = max(1, (Q + kTopSlots - 1) / kTopSlots);
    float lmax = ninf, gcur = ninf;
    constexpr int U = 4;
    for (int q0 = 0; q0 < Q; q0 += U) {
        typename RawT<DT, VEC>::type rg[U], rm[U];
        bool valid[U];
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const long v = (long)(q0 + j) * kTopThreads + tid;
            valid[j] = (q0 + j) < Q && v < nvec;
            if (valid[j]) {
                rg[j] = ld_raw<DT, VEC>(g, v);
                rm[j] = ld_raw<DT, VEC>(sm, v);
            }
        }
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const int q = q0 + j;
            if (q >= Q) break;  // uniform
            if (valid[j]) {
                float hg[VEC], hm[VEC];
                unpack(rg[j], hg);
                unpack(rm[j], hm);
#pragma unroll
                for (int i = 0; i < VEC; ++i) gcur = fmaxf(gcur, fmaf(nbeta, hm[i], hg[i]));
            }
            if ((q + 1) % gsz == 0 || q == Q - 1) {  // uniform: the group is complete
                gm[(q / gsz) * kTopThreads + tid] = gcur;
                lmax = fmaxf(lmax, gcur);
                gcur = ninf;
            }
        }
    }
    float tmax = ninf;  // logits past the last full vector, one per lane of the first lanes
    if (tid < tailc) {
        const long e = nvec * VEC + tid;
        tmax = fmaf(nbeta, ld_elem<DT>(sm, e), ld_elem<DT>(g, e));
        lmax = fmaxf(lmax, tmax);
    }

    // ---- B: a lower bound on the k-th largest logit of the row
    const int per_wave = (topk + kTopWaves - 1) / kTopWaves;
    float bound = lmax - fabsf(lmax) * 2.4e-7f - 1e-37f;  // a real logit of this lane is >= bound
    float wb = ninf;
    for (int t = 0; t < per_wave; ++t) {
        wb = wave_max_f32(bound);
        const unsigned long long holders = __ballot(bound == wb);
        if (holders && lane == first_lane(holders)) bound = ninf;  // take one holder out, keep duplicates
    }
    if (lane == 0) wave_bound[wave] = wb;
    __syncthreads();
    float tau = wave_bound[0];
#pragma unroll
    for (int u = 1; u < kTopWaves; ++u) tau = fminf(tau, wave_bound[u]);
    const float screen = tau - fabsf(tau) * 2.4e-7f - 1e-37f;  // recorded maxima carry fp32 rounding too
    const double tau_d = (double)tau;

    // ---- C: exact values of everything that can still matter
    auto offer = [&](double hc, int idx) {
        if (hc >= tau_d) {
            const int pos = atomicAdd(&cand_count, 1);
            if (pos < kTopCap) {
                c_v[pos] = hc;
                c_i[pos] = idx;
            }
        }
    };
    // The (lane, group) pairs to revisit are few and scattered: they are queued first and then
    // dealt out one per thread, so that all of them are fetched in the same round trip.
    const int nslots = (Q + gsz - 1) / gsz;
    for (int s = 0; s < nslots; ++s) {
        if (gm[s * kTopThreads + tid] >= screen) {
            const int pos = atomicAdd(&todo_count, 1);
            if (pos < kTopTodo) todo[pos] = s * kTopThreads + tid;
        }
    }
    __syncthreads();
    const int ntodo = todo_count;
    if (ntodo > kTopTodo) {  // block-uniform: far too many survivors for the fast path
        __syncthreads();
        topk_by_insertion<DT, VEC>(a, g, sm, oi, ov, c_v, c_i);
        return;
    }
    for (int e = tid; e < ntodo; e += kTopThreads) {
        const int s = todo[e] / kTopThreads, owner = todo[e] % kTopThreads;
        const int qend = min(Q, (s + 1) * gsz);
        for (int q = s * gsz; q < qend; q += 2) {  // two vectors of both rows per round trip
            typename RawT<DT, VEC>::type rg[2], rm[2];
            long v[2];
            bool ok[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                v[j] = (long)(q + j) * kTopThreads + owner;
                ok[j] = q + j < qend && v[j] < nvec;
                if (ok[j]) {
                    rg[j] = ld_raw<DT, VEC>(g, v[j]);
                    rm[j] = ld_raw<DT, VEC>(sm, v[j]);
                }
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                if (!ok[j]) continue;
                float hg[VEC], hm[VEC];
                unpack(rg[j], hg);
                unpack(rm[j], hm);
#pragma unroll
                for (int i = 0; i < VEC; ++i)
                    offer(cloud_logit(hg[i], hm[i], a.beta), (int)(v[j] * VEC) + i);
            }
        }
    }
    if (tid < tailc && tmax >= screen) {
        const long e = nvec * VEC + tid;
        offer(cloud_logit(ld_elem<DT>(g, e), ld_elem<DT>(sm, e), a.beta), (int)e);
    }
    __syncthreads();
    const int M = cand_count;
    if (M > kTopCap) {  // block-uniform: degenerate row, start over on the exact path
        __syncthreads();
        topk_by_insertion<DT, VEC>(a, g, sm, oi, ov, c_v, c_i);
        return;
    }

    // ---- D: rank among the candidates = position in the payload.  A wave takes every 16th
    // candidate; its lanes hold the candidate list in registers (the first 256 entries, normally
    // all of it) and count, together, how many entries precede the wave's candidate.
    constexpr int kHold = 4;
    double hv[kHold];
    int hi[kHold];
#pragma unroll
    for (int j = 0; j < kHold; ++j) {
        const int u = lane + kWave * j;
        hv[j] = u < M ? c_v[u] : -__builtin_huge_val();
        hi[j] = u < M ? c_i[u] : 0x7FFFFFFF;
    }
    for (int i = wave; i < M; i += kTopWaves) {
        const double mv = c_v[i];
        const int mi = c_i[i];
        int cnt = 0;
#pragma unroll
        for (int j = 0; j < kHold; ++j) cnt += beats(hv[j], hi[j], mv, mi) ? 1 : 0;
        for (int u = lane + kWave * kHold; u < M; u += kWave) cnt += beats(c_v[u], c_i[u], mv, mi) ? 1 : 0;
        const int rank = wave_sum_i32(cnt);
        if (lane == 0 && rank < topk) {
            oi[rank] = mi;
            ov[rank] = (float)mv;
        }
    }
}

struct EdgeArgs {
    const int32_t* index;
    const float* value;
    const void* Sp;
    const int32_t* row;
    const float* uniform;
    int32_t* next_token;
    float* next_token_logprob;
    long sb, st;
    int B, kmax, V, topk;
    double beta, T;
    int greedy;
};

__device__ __forceinline__ double wave_max_f64(double x) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) x = fmax(x, __shfl_xor(x, d, kWave));
    return x;
}

template <int DT>
__global__ __launch_bounds__(kEdgeThreads) void edge_resample_kernel(const EdgeArgs a) {
    const int lane = threadIdx.x & 63;
    const int b = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * (kEdgeThreads / kWave) + (threadIdx.x >> 6)));
    if (b >= a.B) return;
    const int r = a.row[b];
    const int idx = lane < a.topk ? a.index[(long)b * a.topk + lane] : -1;
    const bool valid = idx >= 0 && idx < a.V && r >= 0 && r <= a.kmax;
    const unsigned long long vm = __ballot(valid);
    if (vm == 0ull) {
        if (lane == 0) {
            a.next_token[b] = -1;
            if (a.next_token_logprob) a.next_token_logprob[b] = __int_as_float(0x7FC00000);
        }
        return;
    }
    const double ninf = -__builtin_huge_val();
    double h = ninf;
    if (valid) {
        const float hp = ld_elem<DT>(row_ptr<DT>(a.Sp, (long)b * a.sb + (long)r * a.st), idx);
        h = __dadd_rn((double)a.value[(long)b * a.topk + lane], __dmul_rn(a.beta, (double)hp));  // edge adds its term
    }
    const double x = valid ? h / a.T : ninf;
    const double m = wave_max_f64(x);
    const double e = valid ? exp(x - m) : 0.0;
    const double incl_e = wave_incl_scan_f64(e);
    const double lse = m + log(wave_last_f64(incl_e));
    const double lp = valid ? x - lse : ninf;
    const double p = valid ? exp(lp) : 0.0;
    const double cum = wave_incl_scan_f64(p);
    int pick;
    if (a.greedy) {
        const double hm = wave_max_f64(h);
        pick = first_lane(__ballot(valid && h == hm));
    } else {
        const double us = (double)a.uniform[b];
        const unsigned long long over = __ballot(valid && cum > us);
        const unsigned long long pos = __ballot(valid && p > 0.0);
        pick = over ? first_lane(over) : (pos ? 63 - __clzll((long long)pos) : first_lane(vm));
    }
    const int tok = __shfl(idx, pick, kWave);
    const double lpt = __shfl(lp, pick, kWave);
    if (lane == 0) {
        a.next_token[b] = tok;
        if (a.next_token_logprob) a.next_token_logprob[b] = (float)lpt;
    }
}

ss_status check_split_params(const ss_params* p, int32_t topk, long& st, long& sb) {
    if (!p) return SS_ERR_NULL;
    if (p->dtype != SS_F32 && p->dtype != SS_BF16) return SS_ERR_DTYPE;
    if (p->batch < 0 || p->k_max < 0 || p->k_max > SS_MAX_K || p->vocab < 1 || p->vocab > SS_MAX_VOCAB)
        return SS_ERR_SHAPE;
    if (topk < 1 || topk > SS_MAX_TOPK) return SS_ERR_SHAPE;
    if (!std::isfinite(p->beta)) return SS_ERR_PARAM;
    if ((p->flags & ~(uint32_t)SS_FLAG_GREEDY) != 0) return SS_ERR_PARAM;
    if (p->stride_t < 0 || p->stride_b < 0) return SS_ERR_STRIDE;
    st = p->stride_t ? p->stride_t : (long)p->vocab;
    sb = p->stride_b ? p->stride_b : (long)(p->k_max + 1) * st;
    if (st < p->vocab || sb < (long)p->k_max * st + p->vocab) return SS_ERR_STRIDE;
    return SS_OK;
}

}  // namespace

extern "C" {

ss_status specsteer_cloud_topk(const void* G, const void* S_noctx, const int32_t* row, const ss_params* params,
                               int32_t topk, int32_t* out_index, float* out_value, void* stream) {
    long st = 0, sb = 0;
    const ss_status chk = check_split_params(params, topk, st, sb);
    if (chk != SS_OK) return chk;
    if (!G || !S_noctx || !row || !out_index || !out_value) return SS_ERR_NULL;
    if (params->batch == 0) return SS_OK;
    TopArgs a;
    a.G = G; a.Sm = S_noctx; a.row = row; a.out_index = out_index; a.out_value = out_value;
    a.sb = sb; a.st = st; a.B = params->batch; a.kmax = params->k_max; a.V = params->vocab; a.topk = topk;
    a.beta = (double)params->beta;
    const uintptr_t esz = params->dtype == SS_BF16 ? 2 : 4;  // element alignment is all the 16-byte loads need
    if (((reinterpret_cast<uintptr_t>(G) | reinterpret_cast<uintptr_t>(S_noctx)) & (esz - 1)) != 0) return SS_ERR_STRIDE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)params->batch), block(kTopThreads);
    if (params->dtype == SS_BF16)
        hipLaunchKernelGGL((cloud_topk_kernel<SS_BF16, 8>), grid, block, 0, s, a);
    else
        hipLaunchKernelGGL((cloud_topk_kernel<SS_F32, 4>), grid, block, 0, s, a);
    return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_DEVICE;
}

ss_status specsteer_edge_resample(const int32_t* index, const float* value, const void* S_ctx, const int32_t* row,
                                  const float* uniform, const ss_params* params, int32_t topk, int32_t* next_token,
                                  float* next_token_logprob, void* stream) {
    long st = 0, sb = 0;
    const ss_status chk = check_split_params(params, topk, st, sb);
    if (chk != SS_OK) return chk;
    if (!(params->temperature > 0.f) || !std::isfinite(params->temperature)) return SS_ERR_PARAM;
    const bool greedy = (params->flags & SS_FLAG_GREEDY) != 0;
    if (!index || !value || !S_ctx || !row || !next_token || (!greedy && !uniform)) return SS_ERR_NULL;
    if (params->batch == 0) return SS_OK;
    EdgeArgs a;
    a.index = index; a.value = value; a.Sp = S_ctx; a.row = row; a.uniform = uniform; a.next_token = next_token;
    a.next_token_logprob = next_token_logprob; a.sb = sb; a.st = st; a.B = params->batch; a.kmax = params->k_max;
    a.V = params->vocab; a.topk = topk; a.beta = (double)params->beta; a.T = (double)params->temperature;
    a.greedy = greedy ? 1 : 0;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int per = kEdgeThreads / kWave;
    const dim3 grid((unsigned)((params->batch + per - 1) / per)), block(kEdgeThreads);
    if (params->dtype == SS_BF16) hipLaunchKernelGGL((edge_resample_kernel<SS_BF16>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((edge_resample_kernel<SS_F32>), grid, block, 0, s, a);
    return hipGetLastError() == hipSuccess ? SS_OK : SS_ERR_DEVICE;
}

}  // extern "C"
