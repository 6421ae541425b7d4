// libgrpo: token-level GRPO objective with two-sided clipping (INTELLECT-2 paper,
// section 3.4, objective with the bound delta; token-level mean of section 4.1),
// forward and fused backward, hand-written for gfx950 (MI355X).
//
// The path is a streaming reduction over rows of 152k logits: it is bound by HBM
// bandwidth, not by arithmetic, so there is no MFMA here.  The design keeps one
// whole row resident in the vector registers of one workgroup (304 KB of the CU's
// 512 KB register file for a 152064-wide bf16 row: 512 lanes with 256 registers each,
// 152 of them the row), so that the row is
// read from HBM once, reduced twice (max, sum of exponentials) out of registers,
// and the gradient is produced from the same registers: 1 read + 1 write of HBM
// traffic per row instead of 2 reads + 1 write.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdint>

#include "grpo.h"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr unsigned kNegInfF32 = 0xff800000u;
constexpr unsigned kNegInfBf16x2 = 0xff80ff80u;

constexpr int kFlagClipHigh = 1, kFlagClipLow = 2, kFlagDelta = 4, kFlagOutOfBand = 8;

// First 256 bytes of the caller's workspace.
struct WsHeader {
    double D;      // denominator of the token-level mean
    double inv_D;  // 1 / D, or 0 when D == 0
    long long M;   // rows with mask != 0
    int error;     // sticky data-error word (bit 0: token id out of range)
    unsigned fin_ticket;  // blocks of grpo_finalize that have delivered their partial sums
    unsigned live_fill, masked_fill;  // entries grpo_order_rows has reserved at either end of the order array
};
// The row queue: up to kQueueParts counters, each on a 128-byte line of its own, follow
// the 256-byte header.  With P counters in use, counter q hands out the rows q, q + P,
// q + 2P, ...  One counter for the whole GPU sustains only some 15-25 million increments
// a second under contention (measured): enough for 300 KB rows (8 million rows a second),
// not for 64 KB rows.  Narrow rows therefore use eight interleaved partitions, each
// started on by an eighth of the workgroups and then stolen from in turn, which keeps
// single-row granularity; wide rows use one counter, which measured 4-6 % faster there.
constexpr int kFinSegment = 4096;  // rows one workgroup of grpo_finalize / grpo_order_rows takes: four per lane
constexpr int kQueueParts = 8;
constexpr int kQueueStride = 16;  // in unsigned long long: 128 bytes
constexpr size_t kHeaderBytes = 256 + (size_t)kQueueParts * kQueueStride * 8;
__device__ __forceinline__ unsigned long long *queue_counters(WsHeader *hdr)
{
    return (unsigned long long *)((char *)hdr + 256);
}
constexpr long long kMaxVocab = 1ll << 28;  // byte offsets inside a row stay below 2^32

struct RowParams {
    const void *logits;
    void *grad;  // may alias logits: deliberately no __restrict__ anywhere
    const long long *tokens;
    const float *old_lp;
    const float *adv;
    const unsigned char *mask;
    float *logprobs_out;
    float *J_ws;
    unsigned char *flags_ws;
    WsHeader *hdr;
    long long n_tokens, vocab, row_stride;
    float k;      // log2(e) / T: exponents are kept in base 2 for v_exp_f32
    float inv_T;  // 1 / T
    float lo, hi, delta, grad_scale;
    int bwd;  // 0: log-probs only (grpo_logprobs_fwd), 1: objective + gradient
    const int *order;  // optional: the rows in the order they are handed out (grpo_order_rows), else 0, 1, 2, ...
    int queue_chunk;  // rows taken from the queue per increment
    int queue_parts;  // counters in use (1 or kQueueParts)
    // auxiliary terms (kernels instantiated with AUX only)
    const float *ref_lp;  // reference-policy log-probs, or NULL (no KL term)
    const float *token_w; // per-token weights omega_t, or NULL (all ones); 0 = masked row
    float *KL_ws, *H_ws;  // per-row KL estimate and entropy
    float *entropy_out;   // optional copy of the per-row entropy for the caller
    float kl_coef, ent_coef;
};

template <grpo_dtype DT>
struct Elem;
template <>
struct Elem<GRPO_BF16> {
    static constexpr int EPV = 8, BYTES = 2;
};
template <>
struct Elem<GRPO_F32> {
    static constexpr int EPV = 4, BYTES = 4;
};

// Tunables, with the settings measured best on MI355X (5 GB to 20 GB of logits):
//  - non-temporal loads and stores for the two row streams: every byte is touched
//    once, so nothing is gained by keeping it in L2 / Infinity Cache
//    (log-probs pass 5.5 -> 6.3 TB/s, mixed batches about 4% faster).
#ifndef GRPO_NT_LOAD
#define GRPO_NT_LOAD 1
#endif
#ifndef GRPO_NT_STORE
#define GRPO_NT_STORE 1
#endif
// 16-byte global accesses of the row streams.
__device__ __forceinline__ u32x4 ld16(const char *p)
{
#if GRPO_NT_LOAD
    return __builtin_nontemporal_load((const u32x4 *)p);
#else
    return *(const u32x4 *)p;
#endif
}
__device__ __forceinline__ void st16(char *p, const u32x4 &v)
{
#if GRPO_NT_STORE
    __builtin_nontemporal_store(v, (u32x4 *)p);
#else
    *(u32x4 *)p = v;
#endif
}

__device__ __forceinline__ float as_f32(unsigned u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ unsigned as_u32(float f) { return __builtin_bit_cast(unsigned, f); }

// 16-byte vector -> EPV floats.  A bf16 is the upper half of a binary32.
template <grpo_dtype DT>
__device__ __forceinline__ void unpack(const u32x4 &v, float (&f)[Elem<DT>::EPV])
{
    if constexpr (DT == GRPO_BF16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = as_f32(v[i] << 16);
            f[2 * i + 1] = as_f32(v[i] & 0xffff0000u);
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = as_f32(v[i]);
    }
}

// EPV floats -> 16-byte vector; bf16 rounds to nearest even (v_cvt_pk_bf16_f32).
template <grpo_dtype DT>
__device__ __forceinline__ u32x4 pack(const float (&f)[Elem<DT>::EPV])
{
    u32x4 v;
    if constexpr (DT == GRPO_BF16) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f32x2 p = {f[2 * i], f[2 * i + 1]};
            v[i] = __builtin_bit_cast(unsigned, __builtin_convertvector(p, bf16x2));
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = as_u32(f[i]);
    }
    return v;
}

template <grpo_dtype DT>
__device__ __forceinline__ float load_elem(const char *row, long long j)
{
    if constexpr (DT == GRPO_BF16)
        return as_f32((unsigned)((const unsigned short *)row)[j] << 16);
    else
        return ((const float *)row)[j];
}

template <grpo_dtype DT>
__device__ __forceinline__ void store_elem(char *row, long long j, float x)
{
    if constexpr (DT == GRPO_BF16) {
        f32x2 p = {x, 0.f};
        unsigned u = __builtin_bit_cast(unsigned, __builtin_convertvector(p, bf16x2));
        ((unsigned short *)row)[j] = (unsigned short)(u & 0xffffu);
    } else {
        ((float *)row)[j] = x;
    }
}

template <grpo_dtype DT>
__device__ __forceinline__ u32x4 neg_inf_vec()
{
    unsigned w = (DT == GRPO_BF16) ? kNegInfBf16x2 : kNegInfF32;
    u32x4 v = {w, w, w, w};
    return v;
}

// Vector number v of a row: full vectors come as one 16-byte load; the ragged last
// vector (vocab not a multiple of EPV) is gathered element by element and padded
// with -inf, which contributes exp2(-inf) = 0 and never wins the max; vectors past
// the row are all -inf.
template <grpo_dtype DT>
__device__ __forceinline__ u32x4 load_vec(const char *row, int v, int nvec_full, int tail)
{
    constexpr int EPV = Elem<DT>::EPV;
    if (v < nvec_full) return ld16(row + (unsigned)v * 16u);
    u32x4 out = neg_inf_vec<DT>();
    if (v == nvec_full && tail) {
        float f[EPV];
#pragma unroll
        for (int i = 0; i < EPV; ++i)
            f[i] = (i < tail) ? load_elem<DT>(row, (long long)v * EPV + i) : -INFINITY;
        out = pack<DT>(f);  // exact: the values are already representable
    }
    return out;
}

template <grpo_dtype DT>
__device__ __forceinline__ void store_vec(char *row, int v, int nvec_full, int tail,
                                          const float (&g)[Elem<DT>::EPV])
{
    constexpr int EPV = Elem<DT>::EPV;
    if (v < nvec_full) {
        st16(row + (unsigned)v * 16u, pack<DT>(g));
    } else if (v == nvec_full && tail) {
#pragma unroll
        for (int i = 0; i < EPV; ++i)
            if (i < tail) store_elem<DT>(row, (long long)v * EPV + i, g[i]);
    }
}

template <grpo_dtype DT, int BLOCK>
__device__ __forceinline__ void zero_row(char *row, int nvec_full, int tail, int tid)
{
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (int v = tid; v < nvec_full; v += BLOCK) st16(row + (unsigned)v * 16u, z);
    if (tail && tid < tail) store_elem<DT>(row, (long long)nvec_full * Elem<DT>::EPV + tid, 0.f);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load and store of the wavefront, which would drain the gradient
// stores of the previous row and the prefetch of the next one at each of the three
// barriers a row needs.  Nothing in the row kernels passes data between lanes through
// global memory, so LDS ordering is all the barrier has to provide.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---- reductions: data-parallel-primitive (DPP) steps inside the 64-lane wavefront, LDS
// across waves, always in the same order, so results are bitwise reproducible ----
// A DPP step costs a few cycles; the same reduction through ds_bpermute took six round
// trips to LDS of about a hundred cycles each, in front of a workgroup barrier every time.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float identity, float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, identity),
                                                                   __builtin_bit_cast(int, v), CTRL, ROW_MASK,
                                                                   0xf, false));
}
// Quad swaps, mirror inside 8, mirror inside 16: every lane of a row of 16 holds the row's
// result; then lane 15 of a row is added into the next row (rows 1 and 3), lane 31 into
// rows 2 and 3, and lane 63, which has seen everything, is read out for all.
__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_move<0xB1, 0xf>(v, v));
    v = fmaxf(v, dpp_move<0x4E, 0xf>(v, v));
    v = fmaxf(v, dpp_move<0x141, 0xf>(v, v));
    v = fmaxf(v, dpp_move<0x140, 0xf>(v, v));
    v = fmaxf(v, dpp_move<0x142, 0xa>(-INFINITY, v));
    v = fmaxf(v, dpp_move<0x143, 0xc>(-INFINITY, v));
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_move<0xB1, 0xf>(0.f, v);
    v += dpp_move<0x4E, 0xf>(0.f, v);
    v += dpp_move<0x141, 0xf>(0.f, v);
    v += dpp_move<0x140, 0xf>(0.f, v);
    v += dpp_move<0x142, 0xa>(0.f, v);
    v += dpp_move<0x143, 0xc>(0.f, v);
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ long long wave_sum(long long v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// The caller guarantees a __syncthreads() between the reads of one call and the
// writes of the next call on the same LDS array (the other reduction sits between).
template <int BLOCK>
__device__ __forceinline__ float block_max(float v, float *lds)
{
    constexpr int NW = BLOCK / 64;
    v = wave_max(v);
    if constexpr (NW == 1) return v;
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    lds_barrier();
    float r = lds[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) r = fmaxf(r, lds[i]);
    return r;
}
template <int BLOCK>
__device__ __forceinline__ float block_sum(float v, float *lds)
{
    constexpr int NW = BLOCK / 64;
    v = wave_sum(v);
    if constexpr (NW == 1) return v;
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = v;
    lds_barrier();
    float r = lds[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) r += lds[i];
    return r;
}

// Exponents (log2 units) are kept above this floor before they are multiplied by their
// probability: an element at -inf has probability 0 and must contribute 0 to
// sum p log p, not 0 * inf = NaN.  2^-1e30 is 0 all the same.
constexpr float kExpFloor = -1.0e30f;

// Two sums behind one barrier.
template <int BLOCK>
__device__ __forceinline__ void block_sum2(float &a, float &b, float *lds_a, float *lds_b)
{
    constexpr int NW = BLOCK / 64;
    a = wave_sum(a);
    b = wave_sum(b);
    if constexpr (NW == 1) return;
    if ((threadIdx.x & 63) == 0) {
        lds_a[threadIdx.x >> 6] = a;
        lds_b[threadIdx.x >> 6] = b;
    }
    lds_barrier();
    a = lds_a[0];
    b = lds_b[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) {
        a += lds_a[i];
        b += lds_b[i];
    }
}

// Per-row scalars once the row statistics are known.
//   mk     = (max_j z_j) * k                      (k = log2 e / T)
//   s_excl = sum_{j != y} exp2(z_j k - mk)        (the sampled token is left out so that
//            1 - p_y = s_excl / s keeps its precision on near-one-hot rows, where
//            1 - p_y cancels to nothing in fp32)
// Produces l = log pi(y), the bracketed surrogate term J of section 3.4, its
// indicator bits, and c = grad_scale * dloss/dl.
struct RowScalars {
    float logp, J, c, shift, s, s_excl;
    int flags;
    // auxiliary terms: b = weight of -H in the gradient, q2 and bq the two constants of
    // the fused gradient g_j = p_j (q2 + bq a'_j), gy_ent the entropy part of g_y
    float b, q2, bq, gy_ent, mx, log2s;
};

// Scalar transcendental functions of the once-per-row arithmetic, built on the
// hardware's base-2 exponential and logarithm (1 ulp each).  The library versions are
// exact to the last bit but need dozens of registers at the one point of the kernel
// where the whole row is resident; the per-row quantities need 1e-6, not 1e-8.
__device__ __forceinline__ float hw_exp(float x) { return __builtin_amdgcn_exp2f(x * kLog2e); }
__device__ __forceinline__ float hw_log(float x) { return __builtin_amdgcn_logf(x) * kLn2; }
// ln(1 + x), x >= 0: the series below 1/32 (next term x^7/7 < 5e-12), else the logarithm
__device__ __forceinline__ float hw_log1p(float x)
{
    const float series = x * (1.f + x * (-0.5f + x * (1.f / 3 + x * (-0.25f + x * (0.2f - x * (1.f / 6))))));
    return x < 0.03125f ? series : hw_log(1.f + x);
}
// exp(d) - 1: the series below |d| = 0.1 (next term d^8/40320), else the exponential
__device__ __forceinline__ float hw_expm1(float d)
{
    const float series = d * (1.f + d * (0.5f + d * (1.f / 6 + d * (1.f / 24 + d * (1.f / 120 +
                         d * (1.f / 720 + d * (1.f / 5040)))))));
    return fabsf(d) < 0.1f ? series : hw_exp(d) - 1.f;
}

// J, dJ/dl and the indicator bits of the bracketed surrogate term of section 3.4.
__device__ __forceinline__ void surrogate(const RowParams &p, float r, float A, float &J, float &dJ,
                                          int &fl)
{
    // J = min( min(r, delta) A , clip(r, 1 - eps_low, 1 + eps_high) A )
    const float s1 = fminf(r, p.delta) * A;
    const float s2 = fminf(fmaxf(r, p.lo), p.hi) * A;
    const bool first = s1 <= s2;
    J = first ? s1 : s2;
    // dJ/dl = r dJ/dr; a ratio exactly on a boundary counts as not clipped
    const bool open = first ? (r <= p.delta) : (r >= p.lo && r <= p.hi);
    dJ = open ? A * r : 0.f;
    if (r != r || A != A) {  // fminf/fmaxf drop NaNs: put them back
        J = NAN;
        dJ = NAN;
    }
    fl = 0;
    if (A > 0.f && r > p.hi) fl |= kFlagClipHigh;
    if (A < 0.f && r < p.lo) fl |= kFlagClipLow;
    if (A < 0.f && r > p.delta) fl |= kFlagDelta;
    if (r < p.lo || r > p.hi) fl |= kFlagOutOfBand;
}

__device__ __forceinline__ RowScalars row_scalars(const RowParams &p, long long row, float zy,
                                                  float mk, float s_excl)
{
    RowScalars o = {};
    const float ay = fmaf(zy, p.k, -mk);
    // A sum that is not finite has no logarithm: NaN, so that the row is poisoned whatever way
    // a +inf logit came in (with +inf as the row's maximum inf - inf has already made it NaN).
    const float s0 = s_excl + __builtin_amdgcn_exp2f(ay);
    const float s = s0 < INFINITY ? s0 : NAN;
    const float log2s = __builtin_amdgcn_logf(s);
    o.s = s;
    o.s_excl = s_excl;
    o.shift = mk + log2s;
    o.logp = (ay - log2s) * kLn2;
    if (!p.bwd) return o;

    float dJ;
    surrogate(p, hw_exp(o.logp - p.old_lp[row]), p.adv[row], o.J, dJ, o.flags);
    o.c = -(p.grad_scale * dJ) * (float)p.hdr->inv_D;
    return o;
}

// The same with the auxiliary terms (sampled-token KL estimator against a reference
// policy, entropy bonus).  w_excl = sum_{j != y} e_j a_j with a_j = z_j k - mk (log2
// units), a_j = (z_j - max) k here, and e_j = exp2(a_j).
//   H = ln s - ln2 * (sum_j e_j a_j) / s            entropy of softmax(z / T)
//   kl = exp(d) - d - 1, d = l_ref - l              dkl/dl = 1 - exp(d)
//   total gradient: g_j = (c/T)(1[j=y] - p_j) + (b/T) p_j (ln p_j + H)
// where ln p_j + H = ln2 (a_j - Abar), Abar = (sum e a)/s: the normaliser cancels, so
// the entropy part needs no difference of nearly equal numbers even when p_max -> 1.
__device__ __forceinline__ RowScalars row_scalars_aux(const RowParams &p, long long row, float zy,
                                                      float mx, float s_excl, float w_excl,
                                                      float &kl_out, float &H_out)
{
    RowScalars o = {};
    const float ay = (zy - mx) * p.k;
    const float e_y = __builtin_amdgcn_exp2f(ay);
    const float s = s_excl + e_y;
    float ln_s;
    if (e_y > s_excl) {  // the sampled token dominates: ln(1 + x) form keeps l accurate
        const float t = hw_log1p(s_excl / e_y);
        ln_s = fmaf(ay, kLn2, t);
        o.logp = -t;
    } else {
        ln_s = hw_log(s);
        o.logp = fmaf(ay, kLn2, -ln_s);
    }
    const float log2s = ln_s * kLog2e;
    o.s = s;
    o.s_excl = s_excl;
    o.mx = mx;
    o.log2s = log2s;
    const float ay_f = fmaxf(ay, kExpFloor);
    const float abar = fmaf(e_y, ay_f, w_excl) / s;
    const float H = fmaf(-kLn2, abar, ln_s);

    float dJ;
    surrogate(p, hw_exp(o.logp - p.old_lp[row]), p.adv[row], o.J, dJ, o.flags);
    float kl = 0.f, dkl = 0.f;
    if (p.ref_lp) {
        const float d = p.ref_lp[row] - o.logp;
        const float em1 = hw_expm1(d);
        dkl = -em1;
        // exp(d) - d - 1: below |d| = 0.1 the difference cancels, the series does not
        const float series = d * d * (0.5f + d * (1.f / 6 + d * (1.f / 24 + d * (1.f / 120 +
                             d * (1.f / 720 + d * (1.f / 5040))))));
        kl = fabsf(d) < 0.1f ? series : em1 - d;
    }
    // omega_t / D: the weight of this row in all three sums
    const float wD = (p.token_w ? p.token_w[row] : 1.f) * (float)p.hdr->inv_D;
    o.c = (p.grad_scale * (-dJ + p.kl_coef * dkl)) * wD;
    o.b = (p.grad_scale * p.ent_coef) * wD;
    o.bq = o.b * p.inv_T * kLn2;
    o.q2 = fmaf(o.bq, log2s - abar, -o.c * p.inv_T);
    o.gy_ent = o.bq * ((e_y / s) * (ay_f - abar));
    if (p.token_w) {  // the reductions sum omega_t J_t, omega_t kl_t, omega_t H_t
        const float w = p.token_w[row];
        o.J *= w;
        kl *= w;
    }
    kl_out = kl;
    H_out = H;
    return o;
}

// Overwrites element e of a resident vector with -inf.
template <grpo_dtype DT>
__device__ __forceinline__ void set_neg_inf(u32x4 &v, int e)
{
    if constexpr (DT == GRPO_BF16) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            if (d == (e >> 1))
                v[d] = (e & 1) ? ((v[d] & 0x0000ffffu) | 0xff800000u) : ((v[d] & 0xffff0000u) | 0x0000ff80u);
        }
    } else {
#pragma unroll
        for (int d = 0; d < 4; ++d)
            if (d == e) v[d] = kNegInfF32;
    }
}

// max(a, b, c) as one v_max3_f32.  fmaxf() costs more than it looks: the compiler must first
// quiet a possible signalling NaN in every operand it knows nothing about (one v_max_f32 x, x, x
// each), which doubled the instructions of the maximum pass.  The instruction itself skips quiet
// NaNs like fmaxf and turns a signalling NaN into a quiet NaN result; both are fine here, a
// NaN logit poisons its row in the sum pass in any case.  The operands are never results of
// transcendental instructions (those need a wait state the compiler does not insert for
// inline assembly).
__device__ __forceinline__ float max3_f32(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// The running maximum m joined with the elements of one vector: one v_max3_f32 per 32-bit word
// (two bf16, each widened exactly: the upper one by masking, the lower one by a shift), or per
// two fp32 values.  The maximum is exact, which the entropy gradient of a near-one-hot row needs
// (a difference a_max - Abar of order 1e-8 survives in fp32 only if a_max is exactly zero).
template <grpo_dtype DT>
__device__ __forceinline__ float vec_max_into(float m, const u32x4 &z)
{
    if constexpr (DT == GRPO_BF16) {
#pragma unroll
        for (int d = 0; d < 4; ++d) m = max3_f32(m, as_f32(z[d] & 0xffff0000u), as_f32(z[d] << 16));
    } else {
        m = max3_f32(m, as_f32(z[0]), as_f32(z[1]));
        m = max3_f32(m, as_f32(z[2]), as_f32(z[3]));
    }
    return m;
}

// sum_e exp2(z_e k - mk) over one vector.
template <grpo_dtype DT>
__device__ __forceinline__ float exp_sum_vec(const u32x4 &z, float k, float mk)
{
    constexpr int EPV = Elem<DT>::EPV;
    float f[EPV];
    unpack<DT>(z, f);
    float part = 0.f;
#pragma unroll
    for (int e = 0; e < EPV; ++e) part += __builtin_amdgcn_exp2f(fmaf(f[e], k, -mk));
    return part;
}

// Keeps the instruction scheduler from interleaving the work of different vectors of
// the unrolled row loops: with 76 registers per lane holding the row, there is room
// for the temporaries of one vector at a time, not of several.
#define VECTOR_FENCE() __builtin_amdgcn_sched_barrier(0)

// Makes the compiler forget what it knows about a resident vector.  Without this the
// bf16 -> fp32 widening done in one pass over the row is kept alive for the next pass
// (common-subexpression elimination), which turns 4 registers per vector into 12 and
// spills the row to scratch memory.  Emits no instruction.
__device__ __forceinline__ void forget(u32x4 &v) { asm volatile("" : "+v"(v)); }

// One 32-bit word of a resident vector -> its elements (2 bf16 or 1 f32).
template <grpo_dtype DT>
__device__ __forceinline__ void unpack_word(unsigned w, float (&f)[Elem<DT>::EPV / 4])
{
    if constexpr (DT == GRPO_BF16) {
        f[0] = as_f32(w << 16);
        f[1] = as_f32(w & 0xffff0000u);
    } else {
        f[0] = as_f32(w);
    }
}

// The same, also accumulating sum_e e_e a_e (a = exponent in log2 units, floored so
// that an element at -inf contributes 0).  Word by word, with a scheduling fence between words: the auxiliary
// variants need more temporaries per element and the row leaves room for few.
template <grpo_dtype DT>
__device__ __forceinline__ float exp_sum_vec_aux(u32x4 &z, float k, float mx, float &w)
{
    constexpr int EPW = Elem<DT>::EPV / 4;
    float part = 0.f, partw = 0.f;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        float f[EPW];
        forget(z);  // the widening of word d may not start before this point
        unpack_word<DT>(z[d], f);
#pragma unroll
        for (int e = 0; e < EPW; ++e) {
            // (z - max) k rather than fma(z, k, -max k): exactly 0 at the maximum, which the
            // entropy of a near-one-hot row needs (its sum e a is all cancellation otherwise)
            const float a = fmaxf((f[e] - mx) * k, kExpFloor);
            const float ex = __builtin_amdgcn_exp2f(a);
            part += ex;
            partw = fmaf(ex, a, partw);
        }
        // the running sums must exist here: left alone, the additions drift to the end
        // of the row pass and every product waits for them in a register of its own
        asm volatile("" : "+v"(part), "+v"(partw));
        VECTOR_FENCE();
    }
    w += partw;
    asm volatile("" : "+v"(w));
    return part;
}

// Gradient of one vector with the entropy term fused in: g_j = p_j (q2 + bq a'_j),
// a'_j = (z_j - max) k - log2 s = log2 p_j.  Returns the packed vector.
template <grpo_dtype DT>
__device__ __forceinline__ u32x4 grad_vec_aux(u32x4 &z, float k, float mx, float log2s, float q2,
                                              float bq, bool has_y, int ey, float gy)
{
    constexpr int EPW = Elem<DT>::EPV / 4;
    u32x4 out;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        float f[EPW], g[EPW];
        forget(z);
        unpack_word<DT>(z[d], f);
#pragma unroll
        for (int e = 0; e < EPW; ++e) {
            const float a = fmaxf(fmaf(f[e] - mx, k, -log2s), kExpFloor);
            g[e] = __builtin_amdgcn_exp2f(a) * fmaf(bq, a, q2);
        }
        if (has_y) {
#pragma unroll
            for (int e = 0; e < EPW; ++e)
                if (d * EPW + e == ey) g[e] = gy;
        }
        if constexpr (DT == GRPO_BF16) {
            f32x2 pr = {g[0], g[1]};
            out[d] = __builtin_bit_cast(unsigned, __builtin_convertvector(pr, bf16x2));
        } else {
            out[d] = as_u32(g[0]);
        }
        VECTOR_FENCE();
    }
    return out;
}

// Gradient of one vector: g_j = -(c/T) p_j with p_j = exp2(z_j k - shift), and at
// the sampled token g_y = (c/T) (1 - p_y) = (c/T) s_excl / s.
template <grpo_dtype DT>
__device__ __forceinline__ void grad_vec(const u32x4 &z, float k, float shift, float q, bool has_y,
                                         int ey, float gy, float (&g)[Elem<DT>::EPV])
{
    constexpr int EPV = Elem<DT>::EPV;
    float f[EPV];
    unpack<DT>(z, f);
#pragma unroll
    for (int i = 0; i < EPV; ++i) g[i] = __builtin_amdgcn_exp2f(fmaf(f[i], k, -shift)) * q;
    if (has_y) {
#pragma unroll
        for (int i = 0; i < EPV; ++i)
            if (i == ey) g[i] = gy;
    }
}

__device__ __forceinline__ void write_row_outputs(const RowParams &p, long long row, float logp,
                                                  float J, int flags)
{
    if (p.logprobs_out) p.logprobs_out[row] = logp;
    if (p.bwd) {
        p.J_ws[row] = J;
        p.flags_ws[row] = (unsigned char)flags;
    }
}
__device__ __forceinline__ void write_row_aux(const RowParams &p, long long row, float kl, float H)
{
    if (p.KL_ws) p.KL_ws[row] = kl;
    if (p.H_ws) p.H_ws[row] = p.token_w ? H * p.token_w[row] : H;
    if (p.entropy_out) p.entropy_out[row] = H;
}

// Decides whether a row takes part; handles the rows that do not (masked, or with a
// token id outside the vocabulary).  Returns true when the row must be processed.
template <grpo_dtype DT, int BLOCK>
__device__ __forceinline__ bool row_is_live(const RowParams &p, long long row, int nvec_full,
                                            int tail, long long &y)
{
    bool live = p.mask ? (p.mask[row] != 0) : true;
    if (live && p.token_w) live = p.token_w[row] != 0.f;
    bool bad = false;
    y = 0;
    if (live) {
        y = p.tokens[row];
        if (y < 0 || y >= p.vocab) {
            live = false;
            bad = true;
        }
    }
    if (live) return true;
    if (threadIdx.x == 0) {
        // log-probs-only mode has no error word: a bad token id shows up as NaN
        write_row_outputs(p, row, (bad && !p.bwd) ? NAN : 0.f, 0.f, 0);
        write_row_aux(p, row, 0.f, 0.f);
        if (bad && p.bwd) atomicOr(&p.hdr->error, 1);
    }
    if (p.bwd)
        zero_row<DT, BLOCK>((char *)p.grad + row * p.row_stride * Elem<DT>::BYTES, nvec_full, tail,
                            threadIdx.x);
    return false;
}

// A value every lane holds alike, moved to scalar registers: what is derived from it
// (row base addresses, loop conditions) then stays scalar too.
__device__ __forceinline__ long long uniform(long long v)
{
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)(unsigned long long)v);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)((unsigned long long)v >> 32));
    return (long long)(((unsigned long long)hi << 32) | lo);
}

// Pins program order: whatever is computed from `off` afterwards (the address of the
// next row's load into a slot) cannot be moved above the point where `x` (the last
// value computed from the slot's current contents) exists.  Otherwise the compiler
// starts those loads early into fresh registers and the row no longer fits.  Emits no
// instruction.
template <typename X>
__device__ __forceinline__ void order_after(unsigned &off, X &x)
{
    asm volatile("" : "+v"(off), "+v"(x));
}


// One vector of an online softmax pass: running maximum m (in logit units), sum s of the
// exponentials relative to it and, for the entropy, w = sum e a with a the exponent in log2
// units.  The sampled token's element (has_y, ey) takes part in the maximum only.
template <grpo_dtype DT, bool AUX>
__device__ __forceinline__ void online_vec(const u32x4 &z, bool has_y, int ey, float k, float &m, float &s,
                                           float &w)
{
    constexpr int EPV = Elem<DT>::EPV;
    float f[EPV];
    unpack<DT>(z, f);
    float vm = f[0];
#pragma unroll
    for (int e = 1; e + 1 < EPV; e += 2) vm = max3_f32(vm, f[e], f[e + 1]);
    vm = max3_f32(vm, f[EPV - 1], f[EPV - 1]);  // EPV is even: the last element is still to come
    if (vm > m) {
        // new reference: every exponent so far moves by dlt, every term by 2^dlt
        const float dlt = (m - vm) * k;  // -inf the first time: s and w are 0 and stay 0
        const float sc_ = __builtin_amdgcn_exp2f(dlt);
        if constexpr (AUX) w = (s > 0.f) ? sc_ * fmaf(dlt, s, w) : 0.f;
        s *= sc_;
        m = vm;
    }
    const float mk_t = m * k;
    float part = 0.f, partw = 0.f;
#pragma unroll
    for (int e = 0; e < EPV; ++e) {
        const float a = AUX ? fmaxf((f[e] - m) * k, kExpFloor) : fmaf(f[e], k, -mk_t);
        float ex = __builtin_amdgcn_exp2f(a);
        if (has_y && e == ey) ex = 0.f;
        part += ex;
        if constexpr (AUX) partw = fmaf(ex, a, partw);
    }
    if (m > -INFINITY) {  // all -inf so far: exponents would be NaN
        s += part;
        w += partw;
    }
}

// The online partials (m, s, w) of one lane moved to the row's reference maximum mx.
template <bool AUX>
__device__ __forceinline__ void online_rescale(float m, float s, float w, float mx, float k, float &scaled,
                                               float &scaledw)
{
    const float dlt = (m - mx) * k;
    const float sc_ = __builtin_amdgcn_exp2f(dlt);
    scaled = (m > -INFINITY) ? s * sc_ : 0.f;
    scaledw = (AUX && m > -INFINITY && s > 0.f) ? sc_ * fmaf(dlt, s, w) : 0.f;
}

// Workgroups that share a CU, by instantiation.
constexpr int row_blocks_per_cu(int block, int nv)
{
    // more than 19 slots: the instantiations with 256 registers per lane, 512 lanes per CU
    return block == 1024 ? 1 : nv > 19 ? 512 / block : block == 512 ? 2 : nv >= 16 ? 4 : 8;
}
// How many gradient slots of a row wait before they are stored (see the kernel).  In LDS: as
// many as an equal share of 144 KB of the CU's LDS holds for each workgroup on the CU (a slot
// is 16 bytes per lane), at most all of them.  In registers: only the instantiations with 256
// registers per lane; in the benchmark's (512 lanes x 38 slots, the row takes 152 registers)
// 16 slots is the most the compiler fits without spilling, the others state their number.
#ifndef GRPO_ROW_STASH_KB
#define GRPO_ROW_STASH_KB 144
#endif
#ifndef GRPO_ROW_RSTASH
#define GRPO_ROW_RSTASH 16
#endif
constexpr int row_reg_stash_slots(int block, int nv) { return nv > 19 ? GRPO_ROW_RSTASH : 0; }
// Rows wider than 44 slots of 512 lanes keep 50 slots in registers and up to 18 (8 KB each) in
// LDS, 544 KB together.
#ifndef GRPO_WIDE_NV
#define GRPO_WIDE_NV 50
#endif
#ifndef GRPO_WIDE_RST
#define GRPO_WIDE_RST 0
#endif
constexpr int kWideRegSlots = GRPO_WIDE_NV;
// 1: the lane's number is opaque at every use also where the row fits the registers (the per-slot
// in-range masks are then recomputed instead of kept in scalar registers and spilled to lanes)
#ifndef GRPO_OPAQUE_LANE
#define GRPO_OPAQUE_LANE 1
#endif
#ifndef GRPO_REM_NV
#define GRPO_REM_NV 48
#endif
constexpr int kRemRegSlots = GRPO_REM_NV;  // with a streamed remainder: its loop needs registers too
constexpr int row_stash_slots(int block, int nv, int nl = 0)
{
    const int fit = GRPO_ROW_STASH_KB * 1024 / row_blocks_per_cu(block, nv) / (block * 16) - nl;
    return fit < 0 ? 0 : fit < nv ? fit : nv;
}

// ---------------------------------------------------------------------------
// Register-resident row kernel: requires ceil(vocab / EPV) <= BLOCK * (NV + NL).
// One workgroup per row at a time, rows strided over a persistent grid.
// NL > 0: the row is wider than the registers hold and its last NL slots live in LDS, which
// the loads fill directly (buffer loads with LDS as their target).
// RST >= 0: the number of gradient slots that wait in registers, for the instantiations with
// 256 registers beside the benchmark's width; what LDS the row leaves free holds waiting slots too.
// (Skipping the empty slots of a narrower row with a branch per slot was tried instead of
// several widths: the wait counters are then reset to zero at every join and the gradient
// pass ran 1.5 times as long.)
// REM: the row may be wider still; what lies beyond slot NV + NL is streamed from memory, once
// for an online (max, sum) pass that is merged into the resident part's statistics and once
// more for the gradient: 2 reads + 1 write for that remainder only.
// ---------------------------------------------------------------------------
template <grpo_dtype DT, int BLOCK, int NV, bool AUX, bool TAIL, int NL = 0, int RST = -1, bool REM = false>
// 4 wavefronts per SIMD and 128 registers each; the widest instantiations 2 and 256
__global__ void __launch_bounds__(BLOCK, NV > 19 ? 2 : 4) grpo_rows_cached(RowParams p)
{
    constexpr int EPV = Elem<DT>::EPV;
    constexpr int BYTES = Elem<DT>::BYTES;
    constexpr unsigned SLAB = BLOCK * 16u;  // bytes one pass of the workgroup covers
    static_assert(NL == 0 || !TAIL, "LDS-resident slots come without the ragged-tail slot");
    static_assert(!REM || !TAIL, "the streamed remainder comes without the ragged-tail slot");
    constexpr int RU = AUX ? 2 : 4;  // vectors per lane in flight in the remainder loops (what the registers leave)
    // Gradient vectors of the first STASH slots wait in LDS (each lane its own 16 bytes per
    // slot, no sharing), those of the next RSTASH slots in registers, and all of them are
    // stored after the loop over the slots, so that the next row's loads stand in front of
    // them in the memory queue.  Loads and stores retire in issue order: with a store in
    // front of every load the last load returns when everything is done, and the row
    // statistics that follow run with nothing in flight; with the stores behind the loads
    // they drain during that arithmetic (what a row whose gradient is zero gets for free: it
    // issues all loads, then all stores).
    constexpr int STASH = row_stash_slots(BLOCK, NV, NL);
    // further slots that wait in registers
    constexpr int RSTASH = RST < 0 ? row_reg_stash_slots(BLOCK, NV) : RST < NV - STASH ? RST : NV - STASH;
    static_assert(STASH + RSTASH <= NV, "more waiting slots than register slots");
    extern __shared__ __attribute__((aligned(16))) char row_stash[];
    char *const grad_stash = row_stash + (size_t)NL * SLAB;  // behind the LDS-resident part of the row
    __shared__ float lds_max[BLOCK / 64];
    __shared__ float lds_sum[BLOCK / 64];
    __shared__ float lds_sumw[BLOCK / 64];
    __shared__ long long lds_row[2];
    const int tid = threadIdx.x;
    const unsigned toff = (unsigned)tid * 16u;
    const int nvec_full = (int)(p.vocab / EPV);
    const int tail = (int)(p.vocab % EPV);
    // The ragged last vector (vocab not a multiple of EPV) lives in one extra slot
    // that only the first wavefront carries: lane 0 holds the elements, padded with
    // -inf.  Full rows never enter those branches.
    // (The widest instantiation has no registers to spare for that slot and is built
    // without it; ragged rows of that width take the streaming kernel.)
    const bool tail_wave = TAIL && tail != 0 && tid < 64;

    // ---- which row next ----
    // With a workspace (objective + gradient) rows are handed out through a counter in
    // it, one at a time, to whichever workgroup is free: masked rows cost a third of a
    // live row, and a fixed assignment leaves some workgroups with all the live ones.
    // Without a workspace (log-probs only) rows are strided over the grid.
    const bool queued = p.hdr != nullptr;
    long long strided_next = blockIdx.x;
    unsigned grabs = 0;
    // very narrow rows are also handed out several at a time
    const long long chunk = p.queue_chunk;
    long long chunk_next = 0, chunk_end = 0;  // positions inside the current partition
    // consecutive workgroups sit on different XCDs; dividing by 8 first spreads every
    // partition over all XCDs (tying a partition to one XCD measured 4 % slower)
    const int nparts = p.queue_parts;
    int part = (int)((blockIdx.x / 8) % nparts), parts_done = 0;
    auto grab = [&]() -> long long {
        if (!queued) {
            const long long r = strided_next;
            strided_next += gridDim.x;
            return r;
        }
        for (;;) {
            if (chunk_next < chunk_end) {
                const long long r = part + (long long)nparts * chunk_next++;
                if (r < p.n_tokens) return r;
                chunk_next = chunk_end;  // ran off the end of this partition
            }
            if (parts_done == nparts) return p.n_tokens;
            // two LDS slots used alternately: the barrier of grab k+1 separates the reads
            // of grab k from the write of grab k+2 into the same slot
            const unsigned slot = grabs++ & 1u;
            if (tid == 0)
                lds_row[slot] = (long long)atomicAdd(queue_counters(p.hdr) + part * kQueueStride,
                                                     (unsigned long long)chunk);
            lds_barrier();
            const long long base = uniform(lds_row[slot]);
            if (part + (long long)nparts * base >= p.n_tokens) {
                part = (part + 1) % nparts;  // this partition is exhausted: help with the next
                ++parts_done;
                continue;
            }
            chunk_next = base;
            chunk_end = base + chunk;
        }
    };
    // next row that needs the full treatment; rows that do not (masked, bad token id)
    // are finished on the way
    auto acquire = [&](long long &y) -> long long {
        for (;;) {
            long long r = grab();
            if (r >= p.n_tokens) return p.n_tokens;
            if (p.order) r = uniform((long long)p.order[r]);  // position in the hand-out order -> row
            if (row_is_live<DT, BLOCK>(p, r, nvec_full, tail, y)) return r;
        }
    };

    // slot i of lane tid holds vector i * BLOCK + tid of the resident row: consecutive
    // lanes hold consecutive 16-byte pieces; slots past the end of the row stay -inf
    u32x4 buf[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) buf[i] = neg_inf_vec<DT>();
    u32x4 tbuf = neg_inf_vec<DT>();
    float zy = 0.f;

    // The lane's number and byte offset as the slot loops use them.  In the instantiations with
    // LDS-resident slots they are made opaque at every use: otherwise the compiler keeps the
    // vector number, the store offset and the in-range mask of each of the 60 to 68 slots in
    // registers of their own across the whole row loop, and the row spills.
    auto lane = [&]() __attribute__((always_inline)) {
        int t = tid;
        if constexpr (NL > 0 || GRPO_OPAQUE_LANE) asm volatile("" : "+v"(t));
        return t;
    };
    auto lane_off = [&]() __attribute__((always_inline)) {
        unsigned o = toff;
        if constexpr (NL > 0 || GRPO_OPAQUE_LANE) asm volatile("" : "+v"(o));
        return o;
    };
    unsigned noff = toff;  // byte offset of this lane inside a slab, as used by the refills
    auto fetch_slot = [&](const char *zrow, int i) __attribute__((always_inline)) {
        if (i * BLOCK + lane() < nvec_full) buf[i] = ld16(zrow + (size_t)i * SLAB + noff);
    };
    // LDS-resident slot j (slot NV + j of the row): lane tid owns the 16 bytes at j * SLAB + toff,
    // which is also where the load puts them (wavefront base in M0, 16 bytes per lane).  Lanes
    // past the end of the row load nothing and read their piece as -inf.
    const int wave_lds = __builtin_amdgcn_readfirstlane(tid >> 6) * 1024;
    auto fetch_lds_slot = [&](const char *zrow, int j) __attribute__((always_inline)) {
        if constexpr (NL > 0) {
            if ((NV + j) * BLOCK + lane() < nvec_full) {
                const __amdgpu_buffer_rsrc_t rsrc =
                    __builtin_amdgcn_make_buffer_rsrc((void *)zrow, 0, -1, 0x00020000);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(
                    rsrc, (__attribute__((address_space(3))) void *)(row_stash + (size_t)j * SLAB + wave_lds), 16,
                    (int)((unsigned)(NV + j) * SLAB + noff), 0, 0, GRPO_NT_LOAD ? 2 : 0);
            }
        }
    };
    auto lds_slot = [&](int j, int vy_, int ey_) __attribute__((always_inline)) -> u32x4 {
        // each pass reads the slot anew: with an address the compiler can recognise it keeps the
        // first pass's values of all slots in registers for the later passes, and the row spills
        unsigned off = toff;
        asm volatile("" : "+v"(off));
        u32x4 z = *(const u32x4 *)(row_stash + (size_t)j * SLAB + off);
        const int v = (NV + j) * BLOCK + lane();
        if (v >= nvec_full) z = neg_inf_vec<DT>();
        if (v == vy_) set_neg_inf<DT>(z, ey_);  // the sampled token's logit stays out of the sums
        return z;
    };
    // every load of the row has landed (they retire in order, the LDS-bound ones last)
    auto lds_slots_landed = [&]() {
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0)
        __builtin_amdgcn_sched_barrier(0);
    };
    // (always inlined: as a function of its own it would take the row out of the registers)
    auto fetch_all = [&](const char *zrow) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < NV; ++i) fetch_slot(zrow, i);
#pragma unroll
        for (int j = 0; j < NL; ++j) fetch_lds_slot(zrow, j);
    };
    auto fetch_rest = [&](const char *zrow, long long y) {
        if (tail_wave && tid == 0) tbuf = load_vec<DT>(zrow, nvec_full, nvec_full, tail);
        zy = load_elem<DT>(zrow, y);
    };

    long long y = 0, y_next = 0;
    long long row = acquire(y);
    if (row < p.n_tokens) {
        const char *zrow = (const char *)p.logits + row * p.row_stride * BYTES;
        fetch_all(zrow);
        fetch_rest(zrow, y);
    }

    while (row < p.n_tokens) {
        // Take the following row now: its loads are issued while this row's last pass
        // still computes, into the registers that pass has just finished with.
        const long long next = acquire(y_next);
        const bool has_next = next < p.n_tokens;
        const char *zrow_next = (const char *)p.logits + (has_next ? next : row) * p.row_stride * BYTES;

        const int vy = (int)(y / EPV);
        const int ey = (int)(y % EPV);
        // The sampled token's logit is taken out of the resident row (replaced by -inf):
        // the sum below is then s_excl = sum_{j != y}, which keeps 1 - p_y = s_excl / s
        // accurate on near-one-hot rows where it would cancel to 0 in fp32.  One lane
        // of one wavefront does this once per row.
        if (tid == (vy & (BLOCK - 1)) && vy < nvec_full) {
#pragma unroll
            for (int i = 0; i < NV; ++i)
                if (i == vy / BLOCK) set_neg_inf<DT>(buf[i], ey);
        }
        if (tail_wave && tid == 0 && vy == nvec_full) set_neg_inf<DT>(tbuf, ey);

        // reference maximum over j != y, then joined with z_y
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            forget(buf[i]);
            mx = vec_max_into<DT>(mx, buf[i]);
            VECTOR_FENCE();
        }
        if constexpr (NL > 0) {
            lds_slots_landed();
#pragma unroll
            for (int j = 0; j < NL; ++j) {
                    const u32x4 z = lds_slot(j, vy, ey);
                mx = vec_max_into<DT>(mx, z);
                asm volatile("" : "+v"(mx));  // done with this slot before the next one is read
                VECTOR_FENCE();
            }
        }
        if (tail_wave) mx = vec_max_into<DT>(mx, tbuf);
        // the part of the row that is not resident: online statistics, first read
        const char *zrow_cur = (const char *)p.logits + row * p.row_stride * BYTES;
        float rem_m = -INFINITY, rem_s = 0.f, rem_w = 0.f;
        if constexpr (REM) {
            for (int base = (NV + NL) * BLOCK; base < nvec_full; base += RU * BLOCK) {
                u32x4 z[RU];
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    const int v = base + u * BLOCK + tid;
                    z[u] = neg_inf_vec<DT>();
                    if (v < nvec_full) z[u] = ld16(zrow_cur + (size_t)v * 16);
                }
#pragma unroll
                for (int u = 0; u < RU; ++u) {
                    online_vec<DT, AUX>(z[u], base + u * BLOCK + tid == vy, ey, p.k, rem_m, rem_s, rem_w);
                    VECTOR_FENCE();
                }
            }
            mx = fmaxf(mx, rem_m);
        }
        mx = fmaxf(block_max<BLOCK>(mx, lds_max), zy);
        const float mk = mx * p.k;

        // sum of exponentials over j != y; in log-probs-only mode this is the last use
        // of the row, so the next row is fetched slot by slot behind it
        float acc = 0.f, accw = 0.f;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            forget(buf[i]);
            if constexpr (AUX)
                acc += exp_sum_vec_aux<DT>(buf[i], p.k, mx, accw);
            else
                acc += exp_sum_vec<DT>(buf[i], p.k, mk);
            if (!p.bwd && has_next) {
                order_after(noff, acc);
                fetch_slot(zrow_next, i);
            }
            VECTOR_FENCE();
        }
#pragma unroll
        for (int j = 0; j < NL; ++j) {
            u32x4 z = lds_slot(j, vy, ey);
            if constexpr (AUX)
                acc += exp_sum_vec_aux<DT>(z, p.k, mx, accw);
            else
                acc += exp_sum_vec<DT>(z, p.k, mk);
            asm volatile("" : "+v"(acc));  // done with this slot before the next one is read
            if (!p.bwd && has_next) {
                order_after(noff, acc);  // the slot has been read: its refill may start
                fetch_lds_slot(zrow_next, j);
            }
            VECTOR_FENCE();
        }
        if (tail_wave) {
            if constexpr (AUX)
                acc += exp_sum_vec_aux<DT>(tbuf, p.k, mx, accw);
            else
                acc += exp_sum_vec<DT>(tbuf, p.k, mk);
        }
        if constexpr (REM) {
            float scaled, scaledw;
            online_rescale<AUX>(rem_m, rem_s, rem_w, mx, p.k, scaled, scaledw);
            acc += scaled;
            accw += scaledw;
        }
        const float zy_row = zy;
        if (!p.bwd && has_next) fetch_rest(zrow_next, y_next);
        RowScalars sc;
        if constexpr (AUX) {
            block_sum2<BLOCK>(acc, accw, lds_sum, lds_sumw);
            float kl, H;
            sc = row_scalars_aux(p, row, zy_row, mx, acc, accw, kl, H);
            if (tid == 0) write_row_aux(p, row, kl, H);
        } else {
            const float s_excl = block_sum<BLOCK>(acc, lds_sum);
            sc = row_scalars(p, row, zy_row, mk, s_excl);
        }
        if (tid == 0) write_row_outputs(p, row, sc.logp, sc.J, sc.flags);

        if (p.bwd) {
            char *grow = (char *)p.grad + row * p.row_stride * BYTES;
            if (sc.c == 0.f && (!AUX || sc.b == 0.f)) {
                // the gradient of this row is cut: fetch the next row, then zero-fill
                if (has_next) {
                    fetch_all(zrow_next);
                    fetch_rest(zrow_next, y_next);
                }
                zero_row<DT, BLOCK>(grow, nvec_full, tail, tid);
            } else {
                const float q = -sc.c * p.inv_T;
                const float gy = (sc.c * p.inv_T) * (sc.s_excl / sc.s) + (AUX ? sc.gy_ent : 0.f);
                if constexpr (REM) {
                    // second read of the remainder, before the resident slots: behind their
                    // refills these loads would wait for the whole next row
                    for (int base = (NV + NL) * BLOCK; base < nvec_full; base += RU * BLOCK) {
                        u32x4 z[RU];
#pragma unroll
                        for (int u = 0; u < RU; ++u) {
                            const int v = base + u * BLOCK + tid;
                            z[u] = neg_inf_vec<DT>();
                            if (v < nvec_full) z[u] = ld16(zrow_cur + (size_t)v * 16);
                        }
#pragma unroll
                        for (int u = 0; u < RU; ++u) {
                            const int v = base + u * BLOCK + tid;
                            u32x4 packed;
                            if constexpr (AUX) {
                                packed = grad_vec_aux<DT>(z[u], p.k, sc.mx, sc.log2s, sc.q2, sc.bq, v == vy, ey, gy);
                            } else {
                                float g[EPV];
                                grad_vec<DT>(z[u], p.k, sc.shift, q, v == vy, ey, gy, g);
                                packed = pack<DT>(g);
                            }
                            if (v < nvec_full) st16(grow + (size_t)v * 16, packed);
                            VECTOR_FENCE();
                        }
                    }
                }
                u32x4 rstash[RSTASH > 0 ? RSTASH : 1];
#pragma unroll
                for (int i = 0; i < NV; ++i) {
                            const int v = i * BLOCK + lane();
                    forget(buf[i]);
                    u32x4 packed;
                    if constexpr (AUX) {
                        packed = grad_vec_aux<DT>(buf[i], p.k, sc.mx, sc.log2s, sc.q2, sc.bq, v == vy, ey, gy);
                    } else {
                        float g[EPV];
                        grad_vec<DT>(buf[i], p.k, sc.shift, q, v == vy, ey, gy, g);
                        packed = pack<DT>(g);
                    }
                    order_after(noff, packed);
                    // the slot's gradient waits (LDS, then registers) or, for the last slots, is
                    // stored at once, but in every case behind the next row's load into the slot
                    if (i < STASH) *(u32x4 *)(grad_stash + (size_t)i * SLAB + lane_off()) = packed;
                    if (has_next) fetch_slot(zrow_next, i);
                    if (i >= STASH && i < STASH + RSTASH) rstash[i - STASH < 0 ? 0 : i - STASH] = packed;
                    if (i >= STASH + RSTASH && v < nvec_full) st16(grow + (size_t)i * SLAB + lane_off(), packed);
                    VECTOR_FENCE();
                }
#pragma unroll
                for (int j = 0; j < NL; ++j) {
                            const int v = (NV + j) * BLOCK + lane();
                    u32x4 z = lds_slot(j, -1, 0);
                    u32x4 packed;
                    if constexpr (AUX) {
                        packed = grad_vec_aux<DT>(z, p.k, sc.mx, sc.log2s, sc.q2, sc.bq, v == vy, ey, gy);
                    } else {
                        float g[EPV];
                        grad_vec<DT>(z, p.k, sc.shift, q, v == vy, ey, gy, g);
                        packed = pack<DT>(g);
                    }
                    order_after(noff, packed);  // the slot has been read: its refill may start
                    if (has_next) fetch_lds_slot(zrow_next, j);
                    if (v < nvec_full) st16(grow + (size_t)(NV + j) * SLAB + lane_off(), packed);
                    VECTOR_FENCE();
                }
                if (tail_wave && tid == 0) {
                    float g[EPV];
                    if constexpr (AUX) {
                        const u32x4 pk = grad_vec_aux<DT>(tbuf, p.k, sc.mx, sc.log2s, sc.q2, sc.bq, vy == nvec_full, ey, gy);
                        unpack<DT>(pk, g);  // the tail is stored element by element
                    } else {
                        grad_vec<DT>(tbuf, p.k, sc.shift, q, vy == nvec_full, ey, gy, g);
                    }
                    store_vec<DT>(grow, nvec_full, nvec_full, tail, g);
                }
                if (has_next) fetch_rest(zrow_next, y_next);
#pragma unroll
                for (int i = 0; i < STASH; ++i) {
                    const u32x4 packed = *(const u32x4 *)(grad_stash + (size_t)i * SLAB + lane_off());
                    if (i * BLOCK + lane() < nvec_full) st16(grow + (size_t)i * SLAB + lane_off(), packed);
                }
#pragma unroll
                for (int i = STASH; i < STASH + RSTASH; ++i)
                    if (i * BLOCK + lane() < nvec_full) st16(grow + (size_t)i * SLAB + lane_off(), rstash[i - STASH]);
            }
        }
        row = next;
        y = y_next;
    }
}

// ---------------------------------------------------------------------------
// Streaming row kernel for rows too wide for the register file: an online
// (max, sum) pass and a gradient pass, i.e. 2 reads + 1 write.
// ---------------------------------------------------------------------------
template <grpo_dtype DT, int BLOCK, bool AUX>
__global__ void __launch_bounds__(BLOCK) grpo_rows_streamed(RowParams p)
{
    constexpr int EPV = Elem<DT>::EPV;
    constexpr int BYTES = Elem<DT>::BYTES;
    __shared__ float lds_max[BLOCK / 64];
    __shared__ float lds_sum[BLOCK / 64];
    __shared__ float lds_sumw[BLOCK / 64];
    const int tid = threadIdx.x;
    const int nvec_full = (int)(p.vocab / EPV);
    const int tail = (int)(p.vocab % EPV);
    const int nvec = nvec_full + (tail ? 1 : 0);

    for (long long row = blockIdx.x; row < p.n_tokens; row += gridDim.x) {
        long long y;
        if (!row_is_live<DT, BLOCK>(p, row, nvec_full, tail, y)) continue;
        const char *zrow = (const char *)p.logits + row * p.row_stride * BYTES;
        const float zy = load_elem<DT>(zrow, y);
        const int vy = (int)(y / EPV);
        const int ey = (int)(y % EPV);

        float m = -INFINITY, s = 0.f, w = 0.f;
        for (int v = tid; v < nvec; v += BLOCK) {
            const u32x4 z = load_vec<DT>(zrow, v, nvec_full, tail);
            online_vec<DT, AUX>(z, v == vy, ey, p.k, m, s, w);
        }
        const float mx = fmaxf(block_max<BLOCK>(m, lds_max), zy);
        const float mk = mx * p.k;
        float scaled, scaledw;
        online_rescale<AUX>(m, s, w, mx, p.k, scaled, scaledw);
        RowScalars sc;
        if constexpr (AUX) {
            block_sum2<BLOCK>(scaled, scaledw, lds_sum, lds_sumw);
            if (!(mx > -INFINITY)) scaled = NAN;  // a row of -inf (or NaN) has no softmax
            float kl, H;
            sc = row_scalars_aux(p, row, zy, mx, scaled, scaledw, kl, H);
            if (tid == 0) write_row_aux(p, row, kl, H);
        } else {
            float s_excl = block_sum<BLOCK>(scaled, lds_sum);
            if (!(mx > -INFINITY)) s_excl = NAN;
            sc = row_scalars(p, row, zy, mk, s_excl);
        }
        if (tid == 0) write_row_outputs(p, row, sc.logp, sc.J, sc.flags);
        // the LDS arrays are reused by the next row: one barrier separates this row's
        // reads of lds_sum from the next row's writes of lds_max/lds_sum
        lds_barrier();
        if (!p.bwd) continue;

        char *grow = (char *)p.grad + row * p.row_stride * BYTES;
        if (sc.c == 0.f && (!AUX || sc.b == 0.f)) {
            zero_row<DT, BLOCK>(grow, nvec_full, tail, tid);
            continue;
        }
        const float q = -sc.c * p.inv_T;
        const float gy = (sc.c * p.inv_T) * (sc.s_excl / sc.s) + (AUX ? sc.gy_ent : 0.f);
        for (int v = tid; v < nvec; v += BLOCK) {
            u32x4 z = load_vec<DT>(zrow, v, nvec_full, tail);
            float g[EPV];
            if constexpr (AUX) {
                const u32x4 pk = grad_vec_aux<DT>(z, p.k, sc.mx, sc.log2s, sc.q2, sc.bq, v == vy, ey, gy);
                unpack<DT>(pk, g);  // exact: the values are already rounded
            } else {
                grad_vec<DT>(z, p.k, sc.shift, q, v == vy, ey, gy, g);
            }
            store_vec<DT>(grow, v, nvec_full, tail, g);
        }
    }
}

// ---------------------------------------------------------------------------
// Small kernels around the row kernel
// ---------------------------------------------------------------------------

// Counts the unmasked rows and fixes the denominator before any row is processed.
__global__ void __launch_bounds__(1024) grpo_prepare(const unsigned char *mask,
                                                     const float *token_w, long long n,
                                                     double denom, WsHeader *hdr)
{
    __shared__ long long lds[16];
    long long cnt = 0;
    if (mask && !token_w) {
        // the mask alone: 16 bytes per lane and step between the first and the last 16-byte
        // boundary inside it, single bytes before and after (the counts are integers: any order)
        const long long head = ((16 - (long long)((unsigned long long)mask & 15u)) & 15);
        const long long lead = head < n ? head : n;
        const long long nvec = (n - lead) / 16;
        for (long long i = threadIdx.x; i < lead; i += 1024) cnt += mask[i] ? 1 : 0;
        for (long long v = threadIdx.x; v < nvec; v += 1024) {
            const u32x4 w = *(const u32x4 *)(mask + lead + 16 * v);
#pragma unroll
            for (int d = 0; d < 4; ++d)  // bit 7 of every byte that is not zero, then count them
                cnt += __builtin_popcount((w[d] | ((w[d] & 0x7f7f7f7fu) + 0x7f7f7f7fu)) & 0x80808080u);
        }
        for (long long i = lead + 16 * nvec + threadIdx.x; i < n; i += 1024) cnt += mask[i] ? 1 : 0;
    } else if (mask || token_w) {
        for (long long i = threadIdx.x; i < n; i += 1024)
            cnt += ((!mask || mask[i]) && (!token_w || token_w[i] != 0.f)) ? 1 : 0;
    }
    cnt = wave_sum(cnt);
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = cnt;
    if (threadIdx.x < kQueueParts) queue_counters(hdr)[threadIdx.x * kQueueStride] = 0ull;
    __syncthreads();
    if (threadIdx.x == 0) {
        long long M = 0;
        for (int i = 0; i < 16; ++i) M += lds[i];
        if (!mask && !token_w) M = n;
        const double D = denom > 0.0 ? denom : (double)M;
        hdr->D = D;
        hdr->inv_D = D > 0.0 ? 1.0 / D : 0.0;
        hdr->M = M;
        hdr->error = 0;
        hdr->fin_ticket = 0u;
        hdr->live_fill = 0u;
        hdr->masked_fill = 0u;
    }
}

// The order in which grpo_rows_cached hands out the rows of a batch with masked rows: first the
// rows that take part (mask 1 and weight not 0), then the masked ones, which only need zeros.
// Handed out in index order, masked rows between live ones cost more than their bytes: the same
// rows with the masked ones at the end ran 5 to 8 % faster at V = 152064 (the zero fill of a masked
// row and the read-compute-write cycle of a live row share the memory system badly).
// One workgroup per 4096 rows: an ordered compaction inside the workgroup, a range of the output
// reserved with one atomic per class.  order[0 .. M) are the live rows, order[M .. n) the masked
// ones (written from the end).  Which workgroup gets which range varies from run to run; no
// output depends on the order rows are processed in.
__global__ void __launch_bounds__(1024) grpo_order_rows(const unsigned char *mask, const float *token_w,
                                                       long long n, WsHeader *hdr, int *order)
{
    __shared__ int wave_l[16], wave_m[16];
    __shared__ unsigned base_l, base_m;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const long long r0 = (long long)blockIdx.x * kFinSegment + tid * 4ll;  // four consecutive rows per lane
    bool live[4], valid[4];
    int cl = 0, cm = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const long long r = r0 + e;
        valid[e] = r < n;
        live[e] = valid[e] && (!mask || mask[r] != 0) && (!token_w || token_w[r] != 0.f);
        cl += live[e] ? 1 : 0;
        cm += (valid[e] && !live[e]) ? 1 : 0;
    }
    int il = cl, im = cm;  // inclusive scans inside the wavefront
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int ul = __shfl_up(il, o, 64), um = __shfl_up(im, o, 64);
        if (lane >= o) {
            il += ul;
            im += um;
        }
    }
    if (lane == 63) {
        wave_l[wv] = il;
        wave_m[wv] = im;
    }
    __syncthreads();
    int before_l = 0, before_m = 0, tot_l = 0, tot_m = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        if (w < wv) {
            before_l += wave_l[w];
            before_m += wave_m[w];
        }
        tot_l += wave_l[w];
        tot_m += wave_m[w];
    }
    if (tid == 0) {
        base_l = tot_l ? atomicAdd(&hdr->live_fill, (unsigned)tot_l) : 0u;
        base_m = tot_m ? atomicAdd(&hdr->masked_fill, (unsigned)tot_m) : 0u;
    }
    __syncthreads();
    long long pl = (long long)base_l + before_l + (il - cl);
    long long pm = (long long)base_m + before_m + (im - cm);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (live[e])
            order[pl++] = (int)(r0 + e);
        else if (valid[e])
            order[n - 1 - pm++] = (int)(r0 + e);
    }
}

// Log-probs-only calls that bring a workspace use it for the row queue alone.
__global__ void grpo_reset_queue(WsHeader *hdr)
{
    if (threadIdx.x < kQueueParts) queue_counters(hdr)[threadIdx.x * kQueueStride] = 0ull;
    if (threadIdx.x == 0) {
        hdr->error = 0;
    }
}

// loss = -(1/D) sum_t J_t in fp64 and a fixed order; indicator counts.  With the
// auxiliary arrays (KL_ws, H_ws non-NULL) loss_out has four entries:
// total = policy + kl_coef * mean kl - ent_coef * mean H, policy, mean kl, mean H.
//
// One workgroup per segment of kFinSegment rows: it sums its rows (a fixed assignment of rows to
// lanes, wavefronts combined in order), leaves the partial sums in the workspace and draws a
// ticket; the workgroup that draws the last ticket adds the partials in segment order and writes
// the results.  Which workgroup that is varies from run to run, what it computes does not: the
// sums are bitwise reproducible.  (A single workgroup took 13 us for 16384 rows and 0.1 ms for
// 131072; the segments take about as long as one of them.)
struct FinPartial {
    double s[3];
    long long c[4];
    long long pad;
};
static_assert(sizeof(FinPartial) == 64, "one partial per 64 bytes");
constexpr size_t fin_partials_bytes(long long n)
{
    return (((size_t)((n + kFinSegment - 1) / kFinSegment) * sizeof(FinPartial)) + 255) / 256 * 256;
}

__global__ void __launch_bounds__(1024) grpo_finalize(const float *J_ws, const float *KL_ws,
                                                      const float *H_ws,
                                                      const unsigned char *flags_ws, long long n,
                                                      WsHeader *hdr, FinPartial *partials, float kl_coef,
                                                      float ent_coef, float *loss_out,
                                                      long long *counts_out, int *error_out)
{
    __shared__ double lds_j[16][3];
    __shared__ long long lds_c[16][4];
    __shared__ unsigned lds_ticket;
    const bool aux = KL_ws != nullptr;
    const long long nseg = (n + kFinSegment - 1) / kFinSegment;  // 0 for an empty batch: one block, no rows
    // sums x over the block in a fixed order: lanes inside a wavefront, then the wavefronts in turn
    auto block_totals = [&](double (&sj)[3], long long (&c)[4]) {
#pragma unroll
        for (int q = 0; q < 3; ++q) sj[q] = wave_sum(sj[q]);
#pragma unroll
        for (int q = 0; q < 4; ++q) c[q] = wave_sum(c[q]);
        __syncthreads();  // the arrays may still be read from the previous use
        if ((threadIdx.x & 63) == 0) {
#pragma unroll
            for (int q = 0; q < 3; ++q) lds_j[threadIdx.x >> 6][q] = sj[q];
#pragma unroll
            for (int q = 0; q < 4; ++q) lds_c[threadIdx.x >> 6][q] = c[q];
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 3; ++q) sj[q] = 0.0;
#pragma unroll
        for (int q = 0; q < 4; ++q) c[q] = 0;
#pragma unroll 2  // all 16 at once would read 224 registers' worth of partial sums first, and spill
        for (int w = 0; w < 16; ++w) {  // wavefront by wavefront, in order
#pragma unroll
            for (int q = 0; q < 3; ++q) sj[q] += lds_j[w][q];
#pragma unroll
            for (int q = 0; q < 4; ++q) c[q] += lds_c[w][q];
        }
    };

    double sj[3] = {0.0, 0.0, 0.0};
    long long c[4] = {0, 0, 0, 0};
    auto count = [&](int fl) {
        c[0] += (fl & kFlagClipHigh) ? 1 : 0;
        c[1] += (fl & kFlagClipLow) ? 1 : 0;
        c[2] += (fl & kFlagDelta) ? 1 : 0;
        c[3] += (fl & kFlagOutOfBand) ? 1 : 0;
    };
    // this block's segment: four rows per lane (the arrays start on 256-byte boundaries and a
    // segment is a multiple of four rows), the batch's last n % 4 rows one by one
    const long long seg0 = (long long)blockIdx.x * kFinSegment;
    const long long seg1 = seg0 + kFinSegment < n ? seg0 + kFinSegment : n;
    const long long i = seg0 + threadIdx.x * 4ll;
    if (i + 3 < seg1) {
        const float4 j = *(const float4 *)(J_ws + i);
        sj[0] += (double)j.x;
        sj[0] += (double)j.y;
        sj[0] += (double)j.z;
        sj[0] += (double)j.w;
        if (aux) {
            const float4 kl = *(const float4 *)(KL_ws + i), h = *(const float4 *)(H_ws + i);
            sj[1] += (double)kl.x;
            sj[1] += (double)kl.y;
            sj[1] += (double)kl.z;
            sj[1] += (double)kl.w;
            sj[2] += (double)h.x;
            sj[2] += (double)h.y;
            sj[2] += (double)h.z;
            sj[2] += (double)h.w;
        }
        const unsigned fl4 = *(const unsigned *)(flags_ws + i);
#pragma unroll
        for (int b = 0; b < 4; ++b) count((int)((fl4 >> (8 * b)) & 0xffu));
    } else {
        for (long long r = i; r < seg1; ++r) {  // at most three rows, in one lane of the last segment
            sj[0] += (double)J_ws[r];
            if (aux) {
                sj[1] += (double)KL_ws[r];
                sj[2] += (double)H_ws[r];
            }
            count(flags_ws[r]);
        }
    }
    block_totals(sj, c);
    if (nseg > 1) {
        if (threadIdx.x == 0) {
            FinPartial pt;
#pragma unroll
            for (int q = 0; q < 3; ++q) pt.s[q] = sj[q];
#pragma unroll
            for (int q = 0; q < 4; ++q) pt.c[q] = c[q];
            pt.pad = 0;
            partials[blockIdx.x] = pt;
            __threadfence();  // the partial is visible before the ticket is
            lds_ticket = atomicAdd(&hdr->fin_ticket, 1u);
        }
        __syncthreads();
        if (lds_ticket != (unsigned)(nseg - 1)) return;  // whole workgroup alike
        __threadfence();  // the last ticket: every partial has been delivered; read them afresh
#pragma unroll
        for (int q = 0; q < 3; ++q) sj[q] = 0.0;
#pragma unroll
        for (int q = 0; q < 4; ++q) c[q] = 0;
        for (long long sgm = threadIdx.x; sgm < nseg; sgm += 1024) {  // lane l: segments l, l + 1024, ...
            const volatile FinPartial *pp = partials + sgm;
#pragma unroll
            for (int q = 0; q < 3; ++q) sj[q] += pp->s[q];
#pragma unroll
            for (int q = 0; q < 4; ++q) c[q] += pp->c[q];
        }
        block_totals(sj, c);
    }
    if (threadIdx.x == 0) {
        const double policy = 0.0 - sj[0] * hdr->inv_D;
        if (aux) {
            const double klm = sj[1] * hdr->inv_D, hm = sj[2] * hdr->inv_D;
            loss_out[0] = (float)(policy + (double)kl_coef * klm - (double)ent_coef * hm);
            loss_out[1] = (float)policy;
            loss_out[2] = (float)klm;
            loss_out[3] = (float)hm;
        } else {
            loss_out[0] = (float)policy;
        }
        if (error_out) *error_out = hdr->error;  // every row kernel has finished: the word is final
        if (counts_out) {
            counts_out[GRPO_COUNT_TOKENS] = hdr->M;
            counts_out[GRPO_COUNT_CLIP_HIGH] = c[0];
            counts_out[GRPO_COUNT_CLIP_LOW] = c[1];
            counts_out[GRPO_COUNT_DELTA] = c[2];
            counts_out[GRPO_COUNT_OUT_OF_BAND] = c[3];
        }
    }
}

// One wavefront per group: mean, then spread around the mean, both in fp64.
__global__ void __launch_bounds__(64) grpo_group_adv(const float *rewards, long long n_rollouts,
                                                     const int *offsets, long long n_groups,
                                                     long long group_size, double eps_std, int ddof,
                                                     float *adv_out)
{
    const int lane = threadIdx.x;
    for (long long g = blockIdx.x; g < n_groups; g += gridDim.x) {
        long long b = offsets ? (long long)offsets[g] : g * group_size;
        long long e = offsets ? (long long)offsets[g + 1] : (g + 1) * group_size;
        b = b < 0 ? 0 : (b > n_rollouts ? n_rollouts : b);
        e = e < b ? b : (e > n_rollouts ? n_rollouts : e);
        const long long G = e - b;
        if (G == 0) continue;
        double sum = 0.0;
        for (long long i = b + lane; i < e; i += 64) sum += (double)rewards[i];
        const double mu = wave_sum(sum) / (double)G;
        double ss = 0.0;
        for (long long i = b + lane; i < e; i += 64) {
            const double d = (double)rewards[i] - mu;
            ss += d * d;
        }
        ss = wave_sum(ss);
        const double sigma = (G - ddof > 0) ? sqrt(ss / (double)(G - ddof)) : 0.0;
        const double den = sigma + eps_std;
        for (long long i = b + lane; i < e; i += 64)
            adv_out[i] = den > 0.0 ? (float)(((double)rewards[i] - mu) / den) : 0.f;
    }
}

__global__ void __launch_bounds__(256) grpo_adv_to_tokens(const float *adv, long long n_rollouts,
                                                          const int *rollout_of_token,
                                                          long long n_tokens, float *adv_tok)
{
    for (long long t = (long long)blockIdx.x * 256 + threadIdx.x; t < n_tokens;
         t += (long long)gridDim.x * 256) {
        const int r = rollout_of_token[t];
        adv_tok[t] = (r >= 0 && r < n_rollouts) ? adv[r] : NAN;
    }
}

// r_total = r_task - alpha |l_target - l_y| (section 3.1).  The length difference is formed
// in integers, so it is exact.
__global__ void __launch_bounds__(256) grpo_total_rewards_k(const float *task, const int *len,
                                                            const int *target, long long n,
                                                            float alpha, float *out)
{
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long long)gridDim.x * 256) {
        const long long d = (long long)target[i] - (long long)len[i];
        out[i] = task[i] - alpha * (float)(d < 0 ? -d : d);
    }
}

// Online filter (section 3.3): flags the groups whose rewards are not all equal.  One
// wavefront per group.
__global__ void __launch_bounds__(64) grpo_filter_flag(const float *rewards, long long n_rollouts,
                                                       const int *offsets, long long n_groups,
                                                       long long group_size, unsigned char *keep,
                                                       unsigned char *rollout_keep)
{
    const int lane = threadIdx.x;
    for (long long g = blockIdx.x; g < n_groups; g += gridDim.x) {
        long long b = offsets ? (long long)offsets[g] : g * group_size;
        long long e = offsets ? (long long)offsets[g + 1] : (g + 1) * group_size;
        b = b < 0 ? 0 : (b > n_rollouts ? n_rollouts : b);
        e = e < b ? b : (e > n_rollouts ? n_rollouts : e);
        int differs = 0;
        if (e > b) {
            const float first = rewards[b];
            for (long long i = b + lane; i < e; i += 64) differs |= rewards[i] != first ? 1 : 0;
        }
        differs = __any(differs) ? 1 : 0;
        if (lane == 0) keep[g] = (unsigned char)differs;
        if (rollout_keep)
            for (long long i = b + lane; i < e; i += 64) rollout_keep[i] = (unsigned char)differs;
    }
}

// Ordered compaction of the kept group indices: one workgroup walks the flags in chunks
// of 1024 with a running offset, so the output order is the input order.
__global__ void __launch_bounds__(1024) grpo_filter_compact(const unsigned char *keep, long long n_groups,
                                                            int *kept_groups, int *n_kept)
{
    __shared__ int wave_tot[16];
    __shared__ int base;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    if (tid == 0) base = 0;
    __syncthreads();
    for (long long g0 = 0; g0 < n_groups; g0 += 1024) {
        const long long g = g0 + tid;
        const int k = (g < n_groups && keep[g]) ? 1 : 0;
        int incl = k;  // inclusive scan inside the wavefront
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        if (lane == 63) wave_tot[wv] = incl;
        __syncthreads();
        int before = base;
        for (int w2 = 0; w2 < wv; ++w2) before += wave_tot[w2];
        if (k) kept_groups[before + incl - 1] = (int)g;
        __syncthreads();
        if (tid == 0) {
            int tot = 0;
            for (int w2 = 0; w2 < 16; ++w2) tot += wave_tot[w2];
            base += tot;
        }
        __syncthreads();
    }
    const int total = base;
    for (long long g = total + tid; g < n_groups; g += 1024) kept_groups[g] = -1;
    if (tid == 0) *n_kept = total;
}

// Packed (variable-length) batches: rollout i owns rows [cu[i], cu[i+1]).  First every
// row gets "no rollout, weight 0", then each rollout stamps its range.
__global__ void __launch_bounds__(256) grpo_packed_clear(long long n_tokens, float *weights,
                                                         int *rollout_of_token)
{
    for (long long t = (long long)blockIdx.x * 256 + threadIdx.x; t < n_tokens;
         t += (long long)gridDim.x * 256) {
        if (weights) weights[t] = 0.f;
        if (rollout_of_token) rollout_of_token[t] = -1;
    }
}
__global__ void __launch_bounds__(256) grpo_packed_stamp(const long long *cu, long long n_rollouts,
                                                         long long n_tokens, int sample_level,
                                                         float *weights, int *rollout_of_token)
{
    for (long long i = blockIdx.x; i < n_rollouts; i += gridDim.x) {
        long long b = cu[i], e = cu[i + 1];
        b = b < 0 ? 0 : (b > n_tokens ? n_tokens : b);
        e = e < b ? b : (e > n_tokens ? n_tokens : e);
        const float w = sample_level ? (float)(1.0 / (double)(e - b)) : 1.f;
        for (long long t = b + threadIdx.x; t < e; t += 256) {
            if (weights) weights[t] = w;
            if (rollout_of_token) rollout_of_token[t] = (int)i;
        }
    }
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------

int cu_count()
{
    static std::atomic<int> cached[64];          // zero-initialised; host threads may race here
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

template <grpo_dtype DT, int BLOCK, int NV, bool AUX, bool TAIL, int NL = 0, int RST = -1, bool REM = false>
void launch_cached(const RowParams &p, int blocks_per_cu, hipStream_t st)
{
    long long grid = (long long)cu_count() * blocks_per_cu;
    if (grid > p.n_tokens) grid = p.n_tokens;
    // dynamic LDS: the waiting gradient slots, or the LDS-resident part of the row
    constexpr unsigned lds_bytes = (unsigned)(NL + row_stash_slots(BLOCK, NV, NL)) * BLOCK * 16u;
    if constexpr (lds_bytes > 0) {
        static std::atomic<bool> attr_done[64];  // setting the attribute twice is harmless
        int dev = 0;
        if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64 && !attr_done[dev].load()) {
            if (hipFuncSetAttribute((const void *)grpo_rows_cached<DT, BLOCK, NV, AUX, TAIL, NL, RST, REM>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) == hipSuccess)
                attr_done[dev].store(true);
        }
    }
    hipLaunchKernelGGL((grpo_rows_cached<DT, BLOCK, NV, AUX, TAIL, NL, RST, REM>), dim3((unsigned)grid), dim3(BLOCK),
                       lds_bytes, st, p);
}

#ifndef GRPO_QUEUE_CHUNK_BYTES
#define GRPO_QUEUE_CHUNK_BYTES 32768
#endif
// One line per instantiation of the register-resident row kernel:
//   X(id, BLOCK, NV, TAIL, NL, RST without / with the auxiliary terms, REM, workgroups per CU)
// RST: gradient slots that wait in registers (-1: the instantiation's own rule), what fits beside
// the row; the auxiliary terms need a few registers more.
#define GRPO_ROW_KERNELS(X)                                   \
    X(0, 256, 1, true, 0, -1, -1, false, 8)                   \
    X(1, 256, 4, true, 0, -1, -1, false, 8)                   \
    X(2, 256, 16, true, 0, -1, -1, false, 4)                  \
    X(3, 256, 26, false, 0, 8, 8, false, 2)                   \
    X(4, 256, 32, false, 0, 14, 14, false, 2)                 \
    X(5, 512, 16, true, 0, -1, -1, false, 2)                  \
    X(6, 512, 20, false, 0, 2, 2, false, 1)                   \
    X(7, 1024, 10, true, 0, -1, -1, false, 1)                 \
    X(8, 512, 26, false, 0, 8, 8, false, 1)                   \
    X(9, 512, 32, false, 0, 14, 14, false, 1)                 \
    X(10, 512, 38, false, 0, -1, -1, false, 1)                \
    X(11, 512, 44, false, 0, 10, 8, false, 1)                 \
    X(12, 512, kWideRegSlots, false, 4, GRPO_WIDE_RST, GRPO_WIDE_RST, false, 1)  \
    X(13, 512, kWideRegSlots, false, 10, GRPO_WIDE_RST, GRPO_WIDE_RST, false, 1) \
    X(14, 512, kWideRegSlots, false, 18, GRPO_WIDE_RST, GRPO_WIDE_RST, false, 1) \
    X(15, 512, kRemRegSlots, false, 18, 0, 0, true, 1)
constexpr int kRowStreaming = -1;  // the plan's id for grpo_rows_streamed

// Which kernel serves rows of nvec 16-byte vectors (the last one ragged or not).  Host logic only.
//
// Narrow rows take small workgroups, several per CU (each around 16 slots per lane): the
// phases of different rows then overlap inside a CU and the per-row bookkeeping
// (queue, three barriers, scalar arithmetic) is hidden.  Only rows too wide for that
// use one workgroup per CU: 512 lanes with twice the registers, the spare ones holding
// gradient vectors back behind the next row's loads (1024 lanes with up to 10 slots where
// the ragged-tail slot is needed, which those are built without).
int plan_rows(long long nvec, bool ragged)
{
    if (nvec <= 256 * 1) return 0;
    if (nvec <= 256 * 4) return 1;
    if (nvec <= 256 * 16) return 2;
    // two workgroups of 256 lanes with 256 registers each, every gradient slot waiting behind
    // the loads, are 3 % ahead of two of 512 lanes with 128.  (The log-probs pass alone gains
    // nothing, but it takes the same instantiation: the two entry points then give the same
    // bits, and the ratio of an unchanged policy to itself is exactly 1.)
    if (nvec <= 256 * 26 && !ragged) return 3;
    if (nvec <= 256 * 32 && !ragged) return 4;
    if (nvec <= 512 * 16) return 5;
    if (nvec <= 512 * 20 && !ragged) return 6;  // all 20 gradient slots wait: 18 in LDS, 2 in registers
    if (nvec <= 1024 * 10) return 7;
    if (ragged) return kRowStreaming;
    // 512 lanes with twice the registers, in several widths: the arithmetic of a pass runs over
    // every slot of the instantiation, used or not
    if (nvec <= 512 * 26) return 8;
    if (nvec <= 512 * 32) return 9;
    if (nvec <= 512 * 38) return 10;
    if (nvec <= 512 * 44) return 11;
    // wider than the registers: the last slots of the row live in LDS
    if (nvec <= 512 * (kWideRegSlots + 4)) return 12;
    if (nvec <= 512 * (kWideRegSlots + 10)) return 13;
    if (nvec <= 512 * (kWideRegSlots + 18)) return 14;
    // wider than registers and LDS together: the remainder is read twice, up to as much again
    if (nvec <= 512 * 2 * (kRemRegSlots + 18)) return 15;
    return kRowStreaming;
}

template <grpo_dtype DT, bool AUX>
void launch_rows(const RowParams &p_in, hipStream_t st)
{
    RowParams p = p_in;
    {   // rows per queue increment: 1 from 32 KB per row upwards, more for narrower rows
        const long long row_bytes = p.vocab * Elem<DT>::BYTES;
        long long c = (GRPO_QUEUE_CHUNK_BYTES + row_bytes - 1) / row_bytes;
        p.queue_chunk = (int)(c < 1 ? 1 : (c > 64 ? 64 : c));
        p.queue_parts = row_bytes < 200 * 1024 ? kQueueParts : 1;
    }
    const long long nvec = (p.vocab + Elem<DT>::EPV - 1) / Elem<DT>::EPV;
    switch (plan_rows(nvec, p.vocab % Elem<DT>::EPV != 0)) {
#define GRPO_ROW_CASE(ID, BLOCK, NV, TAIL, NL, RSTP, RSTA, REM, PERCU)                              \
    case ID:                                                                                       \
        static_assert(PERCU == row_blocks_per_cu(BLOCK, NV), "workgroups per CU");                \
        launch_cached<DT, BLOCK, NV, AUX, TAIL, NL, (AUX ? RSTA : RSTP), REM>(p, PERCU, st);      \
        break;
        GRPO_ROW_KERNELS(GRPO_ROW_CASE)
#undef GRPO_ROW_CASE
    default: {
        long long grid = (long long)cu_count() * 2;
        if (grid > p.n_tokens) grid = p.n_tokens;
        hipLaunchKernelGGL((grpo_rows_streamed<DT, 1024, AUX>), dim3((unsigned)grid), dim3(1024), 0, st, p);
    }
    }
}

// The integer a C caller put into an enum parameter.  The C ABI passes enums as ints and a C caller
// may pass any int; in C++ merely reading an enum object that holds no enumerator's value is
// undefined, so the boundary reads the bytes instead and validates the integer.
template <typename E>
int raw_enum(const E &e)
{
    static_assert(sizeof(E) == sizeof(int), "enums of the C ABI are ints");
    int v;
    __builtin_memcpy(&v, &e, sizeof v);
    return v;
}

grpo_status check_logits_args(const void *logits, int dtype, int64_t n_tokens, int64_t vocab,
                              int64_t row_stride, const int64_t *tokens, float temperature)
{
    if (dtype != GRPO_F32 && dtype != GRPO_BF16) return GRPO_ERR_DTYPE;
    if (n_tokens < 0 || vocab <= 0 || vocab > kMaxVocab || row_stride < vocab) return GRPO_ERR_SHAPE;
    if (!(temperature > 0.f) || !std::isfinite(temperature)) return GRPO_ERR_PARAM;
    if (n_tokens == 0) return GRPO_OK;
    if (!logits || !tokens) return GRPO_ERR_NULL;
    const int64_t bytes = dtype == GRPO_BF16 ? 2 : 4;
    if (((uintptr_t)logits & 15u) != 0 || ((row_stride * bytes) & 15) != 0) return GRPO_ERR_ALIGN;
    return GRPO_OK;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
unsigned fin_blocks(int64_t n) { return (unsigned)(n > 0 ? (n + kFinSegment - 1) / kFinSegment : 1); }
// header | J, KL estimate, entropy per row (f32 each) | indicator bits per row (u8) | partial sums per
// segment | the order the rows are handed out in (i32 per row)
constexpr size_t loss_workspace_bytes(long long n)
{
    return kHeaderBytes + 4 * (((size_t)n * 4 + 255) / 256 * 256) + ((size_t)n + 255) / 256 * 256 + fin_partials_bytes(n);
}
constexpr long long kOrderMinRowBytes = 32768;  // narrower rows are handed out several at a time, in index order

grpo_status loss_impl(bool aux, const void *logits, int dtype, int64_t n_tokens, int64_t vocab,
                      int64_t row_stride, const int64_t *tokens, const float *old_logprobs,
                      const float *ref_logprobs, const float *advantages, const uint8_t *mask,
                      const float *token_weights, float eps_low, float eps_high, float delta,
                      float temperature, float kl_coef,
                      float entropy_coef, double denom, float grad_scale, float *loss_out,
                      float *logprobs_out, float *entropy_out, int64_t *counts_out,
                      void *grad_logits, void *workspace, size_t workspace_bytes, void *stream,
                      int32_t *error_out = nullptr)
{
    grpo_status rc = check_logits_args(logits, dtype, n_tokens, vocab, row_stride, tokens, temperature);
    if (rc != GRPO_OK) return rc;
    if (!(eps_low >= 0.f && eps_low <= 1.f) || !(eps_high >= 0.f) || !std::isfinite(eps_high) ||
        !(delta > 1.f + eps_high) || std::isnan(denom) || std::isnan(grad_scale) ||
        !std::isfinite(kl_coef) || !std::isfinite(entropy_coef))
        return GRPO_ERR_PARAM;
    if (!loss_out) return GRPO_ERR_NULL;
    if (n_tokens > 0 && (!old_logprobs || !advantages || !grad_logits)) return GRPO_ERR_NULL;
    if (n_tokens > 0 && kl_coef != 0.f && !ref_logprobs) return GRPO_ERR_NULL;
    if (n_tokens > 0 && ((uintptr_t)grad_logits & 15u) != 0) return GRPO_ERR_ALIGN;
    if (!workspace || ((uintptr_t)workspace & 255u) != 0 ||
        workspace_bytes < grpo_workspace_bytes(n_tokens))
        return GRPO_ERR_WORKSPACE;

    char *ws = (char *)workspace;
    const size_t col = align_up((size_t)n_tokens * 4, 256);
    WsHeader *hdr = (WsHeader *)ws;
    float *J_ws = (float *)(ws + kHeaderBytes);
    float *KL_ws = (float *)(ws + kHeaderBytes + col);
    float *H_ws = (float *)(ws + kHeaderBytes + 2 * col);
    unsigned char *flags_ws = (unsigned char *)(ws + kHeaderBytes + 3 * col);
    FinPartial *partials = (FinPartial *)(ws + kHeaderBytes + 3 * col + align_up((size_t)n_tokens, 256));
    int *order = (int *)((char *)partials + fin_partials_bytes(n_tokens));
    hipStream_t st = (hipStream_t)stream;

    hipLaunchKernelGGL(grpo_prepare, dim3(1), dim3(1024), 0, st, mask, aux ? token_weights : nullptr,
                       (long long)n_tokens, denom, hdr);
    if (n_tokens > 0) {
        RowParams p = {};
        p.logits = logits;
        p.grad = grad_logits;
        p.tokens = (const long long *)tokens;
        p.old_lp = old_logprobs;
        p.adv = advantages;
        p.mask = mask;
        p.logprobs_out = logprobs_out;
        p.J_ws = J_ws;
        p.flags_ws = flags_ws;
        p.hdr = hdr;
        p.n_tokens = n_tokens;
        p.vocab = vocab;
        p.row_stride = row_stride;
        p.inv_T = 1.0f / temperature;
        p.k = (float)((double)kLog2e / (double)temperature);
        p.lo = 1.0f - eps_low;
        p.hi = 1.0f + eps_high;
        p.delta = delta;
        p.grad_scale = grad_scale;
        p.bwd = 1;
        // rows of 32 KB and more, some of them masked: the live rows first, then the masked ones
        if ((mask || (aux && token_weights)) && n_tokens <= 0x7fffffffll &&
            vocab * (dtype == GRPO_BF16 ? 2 : 4) >= kOrderMinRowBytes) {
            p.order = order;
            hipLaunchKernelGGL(grpo_order_rows, dim3(fin_blocks(n_tokens)), dim3(1024), 0, st, mask,
                               aux ? token_weights : (const float *)nullptr, (long long)n_tokens, hdr, order);
        }
        if (aux) {
            p.ref_lp = kl_coef != 0.f ? ref_logprobs : nullptr;
            p.token_w = token_weights;
            p.KL_ws = KL_ws;
            p.H_ws = H_ws;
            p.entropy_out = entropy_out;
            p.kl_coef = kl_coef;
            p.ent_coef = entropy_coef;
            if (dtype == GRPO_BF16)
                launch_rows<GRPO_BF16, true>(p, st);
            else
                launch_rows<GRPO_F32, true>(p, st);
        } else {
            if (dtype == GRPO_BF16)
                launch_rows<GRPO_BF16, false>(p, st);
            else
                launch_rows<GRPO_F32, false>(p, st);
        }
    }
    hipLaunchKernelGGL(grpo_finalize, dim3(fin_blocks(n_tokens)), dim3(1024), 0, st, J_ws,
                       aux ? KL_ws : (const float *)nullptr, H_ws, flags_ws, (long long)n_tokens, hdr, partials,
                       kl_coef, entropy_coef, loss_out, (long long *)counts_out, (int *)error_out);
    return hipGetLastError() == hipSuccess ? GRPO_OK : GRPO_ERR_HIP;
}

// ---------------------------------------------------------------------------
// Built-in scratch for grpo_loss_fwd_bwd_noalloc: the workspace of grpo_loss_fwd_bwd for
// GRPO_NOALLOC_MAX_TOKENS rows as an array in the device image, so that callers that cannot
// allocate (graph capture, serving loops) need not bring one.  Every GPU that loads the
// library holds its own copy at its own address.
// ---------------------------------------------------------------------------
constexpr size_t kScratchBytes = loss_workspace_bytes(GRPO_NOALLOC_MAX_TOKENS);
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// The device address of `scratch` on the current device.  In host code the array's name is
// only a handle for the runtime, not an address a kernel can use: the address comes from
// hipGetSymbolAddress, once per device, with that device current, and is kept per device.
void *scratch_address()
{
    static std::atomic<void *> cached[64];  // zero-initialised; racing host threads store the same value
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    void *ptr = cached[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();  // leave no sticky error behind for the caller's next HIP call
            return nullptr;
        }
        cached[dev].store(ptr, std::memory_order_release);
    }
    return ptr;
}

}  // namespace

extern "C" {

const char *grpo_status_string(grpo_status status)
{
    switch (raw_enum(status)) {
        case GRPO_OK: return "ok";
        case GRPO_ERR_NULL: return "a required pointer is NULL";
        case GRPO_ERR_SHAPE: return "bad shape: negative size, vocab outside [1, 2^28] or row_stride < vocab";
        case GRPO_ERR_DTYPE: return "unknown dtype";
        case GRPO_ERR_ALIGN: return "logits/grad base pointer or row pitch is not 16-byte aligned";
        case GRPO_ERR_PARAM:
            return "bad parameter: need temperature > 0, 0 <= eps_low <= 1, eps_high >= 0, "
                   "delta > 1 + eps_high, eps_std >= 0, ddof in {0,1}";
        case GRPO_ERR_WORKSPACE: return "workspace is NULL, not 256-byte aligned or too small";
        case GRPO_ERR_HIP: return "HIP runtime error at kernel launch";
        case GRPO_ERR_CAPACITY:
            return "n_tokens exceeds GRPO_NOALLOC_MAX_TOKENS, the rows the library's built-in scratch array holds";
    }
    return "unknown status";
}

grpo_status grpo_row_kernel_plan(grpo_dtype dtype_arg, int64_t vocab, grpo_row_plan *plan_out)
{
    const int dtype = raw_enum(dtype_arg);
    if (dtype != GRPO_F32 && dtype != GRPO_BF16) return GRPO_ERR_DTYPE;
    if (vocab <= 0 || vocab > kMaxVocab) return GRPO_ERR_SHAPE;
    if (!plan_out) return GRPO_ERR_NULL;
    const int epv = dtype == GRPO_BF16 ? 8 : 4;
    grpo_row_plan r = {};
    r.vectors = (vocab + epv - 1) / epv;
    switch (plan_rows(r.vectors, vocab % epv != 0)) {
#define GRPO_ROW_CASE(ID, BLOCK, NV, TAIL, NL, RSTP, RSTA, REM, PERCU) \
    case ID:                                                          \
        r.lanes = BLOCK;                                              \
        r.register_slots = NV;                                        \
        r.lds_slots = NL;                                             \
        r.workgroups_per_cu = PERCU;                                  \
        r.ragged_tail_slot = TAIL ? 1 : 0;                            \
        r.streamed_remainder = REM ? 1 : 0;                           \
        break;
        GRPO_ROW_KERNELS(GRPO_ROW_CASE)
#undef GRPO_ROW_CASE
    default:
        r.streaming = 1;
        r.lanes = 1024;
        r.workgroups_per_cu = 2;
    }
    const int64_t capacity = (int64_t)r.lanes * (r.register_slots + r.lds_slots);
    r.resident_vectors = r.streaming ? 0 : (r.vectors < capacity ? r.vectors : capacity);
    *plan_out = r;
    return GRPO_OK;
}

size_t grpo_workspace_bytes(int64_t n_tokens)
{
    if (n_tokens < 0) return 0;
    return loss_workspace_bytes(n_tokens);
}

grpo_status grpo_group_advantages(const float *rewards, int64_t n_rollouts,
                                  const int32_t *group_offsets, int64_t n_groups,
                                  int64_t group_size, float eps_std, int ddof, float *adv_out,
                                  const int32_t *rollout_of_token, int64_t n_tokens,
                                  float *adv_tok_out, void *stream)
{
    if (n_rollouts < 0 || n_groups < 0 || n_tokens < 0) return GRPO_ERR_SHAPE;
    if (!group_offsets && (group_size <= 0 || n_groups * group_size != n_rollouts) && n_groups > 0)
        return GRPO_ERR_SHAPE;
    if (!(eps_std >= 0.f) || !std::isfinite(eps_std) || (ddof != 0 && ddof != 1)) return GRPO_ERR_PARAM;
    if (n_groups > 0 && n_rollouts > 0 && (!rewards || !adv_out)) return GRPO_ERR_NULL;
    if (rollout_of_token && n_tokens > 0 && (!adv_tok_out || !adv_out)) return GRPO_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    const bool any_work = (n_groups > 0 && n_rollouts > 0) || (rollout_of_token && n_tokens > 0);
    if (!any_work) return GRPO_OK;
    if (n_groups > 0 && n_rollouts > 0) {
        const unsigned grid = (unsigned)(n_groups < 4096 ? n_groups : 4096);
        hipLaunchKernelGGL(grpo_group_adv, dim3(grid), dim3(64), 0, st, rewards, (long long)n_rollouts,
                           group_offsets, (long long)n_groups, (long long)group_size, (double)eps_std,
                           ddof, adv_out);
    }
    if (rollout_of_token && n_tokens > 0) {
        long long blocks = (n_tokens + 255) / 256;
        if (blocks > 4096) blocks = 4096;
        hipLaunchKernelGGL(grpo_adv_to_tokens, dim3((unsigned)blocks), dim3(256), 0, st, adv_out,
                           (long long)n_rollouts, rollout_of_token, (long long)n_tokens, adv_tok_out);
    }
    return hipGetLastError() == hipSuccess ? GRPO_OK : GRPO_ERR_HIP;
}

grpo_status grpo_total_rewards(const float *task_rewards, const int32_t *lengths,
                               const int32_t *target_lengths, int64_t n_rollouts, float alpha,
                               float *rewards_out, void *stream)
{
    if (n_rollouts < 0) return GRPO_ERR_SHAPE;
    if (!std::isfinite(alpha)) return GRPO_ERR_PARAM;
    if (n_rollouts == 0) return GRPO_OK;
    if (!task_rewards || !lengths || !target_lengths || !rewards_out) return GRPO_ERR_NULL;
    long long blocks = (n_rollouts + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(grpo_total_rewards_k, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       task_rewards, lengths, target_lengths, (long long)n_rollouts, alpha, rewards_out);
    return hipGetLastError() == hipSuccess ? GRPO_OK : GRPO_ERR_HIP;
}

grpo_status grpo_filter_groups(const float *rewards, int64_t n_rollouts, const int32_t *group_offsets,
                               int64_t n_groups, int64_t group_size, uint8_t *keep_out,
                               int32_t *kept_groups_out, int32_t *n_kept_out,
                               uint8_t *rollout_keep_out, void *stream)
{
    if (n_rollouts < 0 || n_groups < 0 || n_groups > 0x7fffffffll) return GRPO_ERR_SHAPE;
    if (!group_offsets && n_groups > 0 && (group_size <= 0 || n_groups * group_size != n_rollouts))
        return GRPO_ERR_SHAPE;
    if (!n_kept_out) return GRPO_ERR_NULL;
    if (n_groups > 0 && (!keep_out || !kept_groups_out)) return GRPO_ERR_NULL;
    if (n_groups > 0 && n_rollouts > 0 && !rewards) return GRPO_ERR_NULL;
    hipStream_t st = (hipStream_t)stream;
    if (n_groups > 0) {
        const unsigned grid = (unsigned)(n_groups < 4096 ? n_groups : 4096);
        hipLaunchKernelGGL(grpo_filter_flag, dim3(grid), dim3(64), 0, st, rewards, (long long)n_rollouts,
                           group_offsets, (long long)n_groups, (long long)group_size, keep_out,
                           rollout_keep_out);
    }
    hipLaunchKernelGGL(grpo_filter_compact, dim3(1), dim3(1024), 0, st, keep_out, (long long)n_groups,
                       kept_groups_out, n_kept_out);
    return hipGetLastError() == hipSuccess ? GRPO_OK : GRPO_ERR_HIP;
}

grpo_status grpo_packed_layout(const int64_t *cu_seqlens, int64_t n_rollouts, int64_t n_tokens,
                               int sample_level, float *weights_out, int32_t *rollout_of_token_out,
                               void *stream)
{
    if (n_rollouts < 0 || n_tokens < 0 || n_rollouts > 0x7fffffffll) return GRPO_ERR_SHAPE;
    if (n_rollouts > 0 && !cu_seqlens) return GRPO_ERR_NULL;
    if (!weights_out && !rollout_of_token_out) return GRPO_ERR_NULL;
    if (n_tokens == 0) return GRPO_OK;
    hipStream_t st = (hipStream_t)stream;
    long long blocks = (n_tokens + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(grpo_packed_clear, dim3((unsigned)blocks), dim3(256), 0, st, (long long)n_tokens,
                       weights_out, rollout_of_token_out);
    if (n_rollouts > 0) {
        const unsigned grid = (unsigned)(n_rollouts < 4096 ? n_rollouts : 4096);
        hipLaunchKernelGGL(grpo_packed_stamp, dim3(grid), dim3(256), 0, st, (const long long *)cu_seqlens,
                           (long long)n_rollouts, (long long)n_tokens, sample_level ? 1 : 0, weights_out,
                           rollout_of_token_out);
    }
    return hipGetLastError() == hipSuccess ? GRPO_OK : GRPO_ERR_HIP;
}

grpo_status grpo_logprobs_fwd(const void *logits, grpo_dtype dtype_arg, int64_t n_tokens, int64_t vocab,
                              int64_t row_stride, const int64_t *tokens, const uint8_t *mask,
                              float temperature, float *logprobs_out, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    const int dtype = raw_enum(dtype_arg);
    grpo_status rc = check_logits_args(logits, dtype, n_tokens, vocab, row_stride, tokens, temperature);
    if (rc != GRPO_OK) return rc;
    if (workspace && (((uintptr_t)workspace & 255u) != 0 || workspace_bytes < kHeaderBytes))
        return GRPO_ERR_WORKSPACE;
    if (n_tokens == 0) return GRPO_OK;
    if (!logprobs_out) return GRPO_ERR_NULL;
    RowParams p = {};
    p.logits = logits;
    p.tokens = (const long long *)tokens;
    p.mask = mask;
    p.logprobs_out = logprobs_out;
    p.hdr = (WsHeader *)workspace;  // NULL: rows are strided over the grid instead of queued
    p.n_tokens = n_tokens;
    p.vocab = vocab;
    p.row_stride = row_stride;
    p.inv_T = 1.0f / temperature;
    p.k = (float)((double)kLog2e / (double)temperature);
    p.bwd = 0;
    hipStream_t st = (hipStream_t)stream;
    if (workspace) hipLaunchKernelGGL(grpo_reset_queue, dim3(1), dim3(64), 0, st, p.hdr);
    if (dtype == GRPO_BF16)
        launch_rows<GRPO_BF16, false>(p, st);
    else
        launch_rows<GRPO_F32, false>(p, st);
    return hipGetLastError() == hipSuccess ? GRPO_OK : GRPO_ERR_HIP;
}

grpo_status grpo_loss_fwd_bwd(const void *logits, grpo_dtype dtype_arg, int64_t n_tokens, int64_t vocab,
                              int64_t row_stride, const int64_t *tokens, const float *old_logprobs,
                              const float *advantages, const uint8_t *mask, float eps_low,
                              float eps_high, float delta, float temperature, double denom,
                              float grad_scale, float *loss_out, float *logprobs_out,
                              int64_t *counts_out, void *grad_logits, void *workspace,
                              size_t workspace_bytes, void *stream)
{
    const int dtype = raw_enum(dtype_arg);
    return loss_impl(false, logits, dtype, n_tokens, vocab, row_stride, tokens, old_logprobs, nullptr,
                     advantages, mask, nullptr, eps_low, eps_high, delta, temperature, 0.f, 0.f, denom,
                     grad_scale, loss_out, logprobs_out, nullptr, counts_out, grad_logits, workspace,
                     workspace_bytes, stream);
}

grpo_status grpo_loss_fwd_bwd_noalloc(const void *logits, grpo_dtype dtype_arg, int64_t n_tokens,
                                      int64_t vocab, int64_t row_stride, const int64_t *tokens,
                                      const float *old_logprobs, const float *advantages,
                                      const uint8_t *mask, float eps_low, float eps_high,
                                      float delta, float temperature, double denom,
                                      float grad_scale, float *loss_out, float *logprobs_out,
                                      int64_t *counts_out, void *grad_logits, int32_t *error_out,
                                      void *stream)
{
    const int dtype = raw_enum(dtype_arg);
    // the size limit first: it needs no device, and nothing may be launched beyond it
    if (n_tokens > (int64_t)GRPO_NOALLOC_MAX_TOKENS) return GRPO_ERR_CAPACITY;
    static_assert(kScratchBytes % 256 == 0, "the scratch array is a whole number of 256-byte lines");
    // Validate everything else against a stand-in address before the device is asked for the
    // real one, so that argument errors are reported the same way with or without a GPU.
    // (loss_impl launches nothing when validation fails, and fails here only on arguments.)
    if (n_tokens >= 0 && grpo_workspace_bytes(n_tokens) > kScratchBytes) return GRPO_ERR_CAPACITY;
    {
        const grpo_status rc = check_logits_args(logits, dtype, n_tokens, vocab, row_stride, tokens, temperature);
        if (rc != GRPO_OK) return rc;
        if (!(eps_low >= 0.f && eps_low <= 1.f) || !(eps_high >= 0.f) || !std::isfinite(eps_high) ||
            !(delta > 1.f + eps_high) || std::isnan(denom) || std::isnan(grad_scale))
            return GRPO_ERR_PARAM;
        if (!loss_out) return GRPO_ERR_NULL;
        if (n_tokens > 0 && (!old_logprobs || !advantages || !grad_logits)) return GRPO_ERR_NULL;
        if (n_tokens > 0 && ((uintptr_t)grad_logits & 15u) != 0) return GRPO_ERR_ALIGN;
    }
    void *ws = scratch_address();
    if (!ws) return GRPO_ERR_HIP;
    return loss_impl(false, logits, dtype, n_tokens, vocab, row_stride, tokens, old_logprobs, nullptr,
                     advantages, mask, nullptr, eps_low, eps_high, delta, temperature, 0.f, 0.f, denom,
                     grad_scale, loss_out, logprobs_out, nullptr, counts_out, grad_logits, ws,
                     kScratchBytes, stream, error_out);
}

grpo_status grpo_loss_aux_fwd_bwd(const void *logits, grpo_dtype dtype_arg, int64_t n_tokens,
                                  int64_t vocab, int64_t row_stride, const int64_t *tokens,
                                  const float *old_logprobs, const float *ref_logprobs,
                                  const float *advantages, const uint8_t *mask,
                                  const float *token_weights, float eps_low, float eps_high,
                                  float delta, float temperature, float kl_coef,
                                  float entropy_coef, double denom, float grad_scale,
                                  float *loss_out, float *logprobs_out, float *entropy_out,
                                  int64_t *counts_out, void *grad_logits, void *workspace,
                                  size_t workspace_bytes, void *stream)
{
    const int dtype = raw_enum(dtype_arg);
    return loss_impl(true, logits, dtype, n_tokens, vocab, row_stride, tokens, old_logprobs,
                     ref_logprobs, advantages, mask, token_weights, eps_low, eps_high, delta,
                     temperature, kl_coef,
                     entropy_coef, denom, grad_scale, loss_out, logprobs_out, entropy_out, counts_out,
                     grad_logits, workspace, workspace_bytes, stream);
}

grpo_status grpo_workspace_error(const void *workspace, int32_t *flag_out, void *stream)
{
    if (!workspace || !flag_out) return GRPO_ERR_NULL;
    const WsHeader *hdr = (const WsHeader *)workspace;
    int v = 0;
    if (hipMemcpyAsync(&v, &hdr->error, sizeof(int), hipMemcpyDeviceToHost, (hipStream_t)stream) != hipSuccess)
        return GRPO_ERR_HIP;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return GRPO_ERR_HIP;
    *flag_out = v;
    return GRPO_OK;
}

}  // extern "C"

#include "lmhead.hpp"
