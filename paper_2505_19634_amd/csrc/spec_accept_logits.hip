// spec_accept_logits: speculative-sampling acceptance straight from target / draft LOGITS, so
// that the V-wide softmax outputs p and q are never written to memory (for the 32B-shaped
// workload: 34 MB of bf16 logits read instead of 34 MB read + 68 MB written + 13-19 MB re-read).
// The rule is the one of spec_accept (paper Section 2 / 3.2: draft proposes, target verifies,
// losslessly); the distributions are softmax(z * inv_temperature).
//
// To be independent of summation order and of any exp() implementation, the softmax is defined on
// integers: y_v = fp32(z_v) * inv_temp, m = max_v y_v, t_v = (y_v - m) * log2(e),
//   E_v = trunc(P(frac(-t_v)) * 2^(30 - floor(-t_v)))   (0 when floor(-t_v) >= 31),
// P a fixed degree-6 polynomial for 2^-f evaluated with fused multiply-adds, S = sum_v E_v, and the
// probability of v is E_v / S exactly.  Accept x iff U * Eq(x) * Sp < 2^24 * Ep(x) * Sq with
// U = trunc(u * 2^24); residual weights W_v = max(0, Ep_v * Sq - Eq_v * Sp); bonus weights Ep_v;
// token = first v whose prefix sum exceeds floor(U_k * sum W / 2^24).  128-bit integers.
//
// Three launches:
//   lg_max_kernel, lg_sum_kernel   grid (pieces of 16384 logits, B * (2k + 1) rows): piece maxima, then --
//                       with the row maximum known -- the pieces' integer weight sums, added into one
//                       64-bit sum per row with device-scope atomics (integers: any order gives the same
//                       sum); the second sweep of the logits is served by the L2 / memory-side cache.
//   lg_scan_pick_kernel grid (chunks, B): accept tests -> n; 128-bit chunk sums of the weights of row n, published as
//                       six 8-byte words that each carry 32 bits of a sum and this call's tag.  The workgroup of a
//                       branch's LAST chunk then collects the branch's sums (it waits only for workgroups with smaller
//                       block indices, dispatched before it; the wait is bounded) and finds the chunk and the token
//                       where the integer CDF crosses the threshold, re-reading that one chunk.
// Every floating-point operation in this file is rounded on its own, as the definition of the integer weights
// says: the compiler's default for device code would otherwise be free to merge a multiplication and a
// following addition or subtraction into one fused operation (one rounding), depending on how the
// surrounding code happens to be shaped.  Fused multiply-adds are written out where the definition has them.
#pragma clang fp contract(off)
#include "lotts_common.h"

namespace lotts {

typedef unsigned __int128 u128;

constexpr int kLgThreads = 256;
constexpr int kLgWaves = kLgThreads / kWave;
constexpr int kLgPiece = 16384;      // logits per piece of the row statistics (V <= 2^20: at most 64 pieces)
constexpr int kLgChunk = 2048;       // tokens per chunk: 8 per thread
constexpr int kLgMaxChunks = 512;    // V <= 2^20
constexpr int kLgMaxK = kLgThreads;

struct RowStat {
    float m;          // row maximum of y
    float pad;
    unsigned long long S;  // sum of the integer weights
};

// One multiplication / subtraction, rounded to nearest.  Defined here, under the pragma above: the toolkit's
// __fmul_rn / __fsub_rn are plain operators compiled under the default mode, and a product and a difference taken
// through them were merged into one fused operation once the two were inlined next to each other.
__device__ __forceinline__ float mul_rn(float a, float b) { return a * b; }
__device__ __forceinline__ float sub_rn(float a, float b) { return a - b; }

__device__ __forceinline__ float bf16_bits_to_float(unsigned short h) { return __uint_as_float((unsigned)h << 16); }

// 2^30 * 2^-f on [0, 1): the polynomial of the definition (c0 = 1 exactly), fused multiply-adds only, with every
// coefficient scaled by 2^30.  Scaling by a power of two commutes with each rounding (no result comes near the
// ends of the exponent range), so this is 2^30 times the definition's P(f), bit for bit.
__device__ __forceinline__ float pow2_neg_poly_2p30(float f) {
    float g = 0x1.e243bep+16f;
    g = __fmaf_rn(g, f, -0x1.52a284p+20f);
    g = __fmaf_rn(g, f, 0x1.3a7ae4p+23f);
    g = __fmaf_rn(g, f, -0x1.c6a66cp+25f);
    g = __fmaf_rn(g, f, 0x1.ebfbaap+27f);
    g = __fmaf_rn(g, f, -0x1.62e430p+29f);
    g = __fmaf_rn(g, f, 0x1p+30f);
    return g;
}

// E = trunc(2^t * 2^30) through the definition's steps; every operation individually rounded
__device__ __forceinline__ unsigned logit_weight(float y, float m) {
    const float t = mul_rn(sub_rn(y, m), 0x1.715476p+0f);
    // -t clamped to 31 (also for -inf logits and NaN from a row that is -inf throughout: fminf returns
    // the other operand): from 31 on the weight truncates to 0 by itself, P(0) * 2^-1 = 0.5, so the
    // definition's "0 when floor(-t) >= 31" needs no branch and no select
    const float a = fminf(-t, 31.0f);
    // a - floor(a) in one instruction (exact for 0 <= a <= 31, as the subtraction is); floor(a) by truncation
    const float f = __builtin_amdgcn_fractf(a);
    const unsigned n = (unsigned)(int)a;
    // trunc(P * 2^(30 - n)) = trunc(P * 2^30) >> n: P * 2^30 <= 2^30 is a non-negative number, and flooring
    // it before the division by 2^n does not change the floor of the quotient
    return __float2uint_rz(pow2_neg_poly_2p30(f)) >> n;
}

template <bool BF16>
__device__ __forceinline__ float load_y(const void* z, size_t idx, float inv_temp) {
    const float v = BF16 ? bf16_bits_to_float(static_cast<const unsigned short*>(z)[idx])
                         : static_cast<const float*>(z)[idx];
    return mul_rn(v, inv_temp);
}

// 8 consecutive logits starting at a multiple of 8 (rows are 16-byte aligned when V % 8 == 0)
template <bool BF16>
__device__ __forceinline__ void load_y8(const void* z, size_t idx, float inv_temp, float (&y)[8]) {
    if (BF16) {
        const uint4 r = *reinterpret_cast<const uint4*>(static_cast<const unsigned short*>(z) + idx);
        const unsigned w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            y[2 * i] = mul_rn(__uint_as_float(w[i] << 16), inv_temp);
            y[2 * i + 1] = mul_rn(__uint_as_float(w[i] & 0xffff0000u), inv_temp);
        }
    } else {
        const float4 a = *reinterpret_cast<const float4*>(static_cast<const float*>(z) + idx);
        const float4 b = *reinterpret_cast<const float4*>(static_cast<const float*>(z) + idx + 4);
        const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) y[i] = mul_rn(v[i], inv_temp);
    }
}

// A thread's share of one piece of kLgPiece logits: kLgPieceIters groups of 8 consecutive logits, all
// requested before the first is used (one 16-byte load per group would otherwise wait for the one
// before it, and the sweep would run at the memory latency instead of the bandwidth).  Groups past
// the end of the row read as -inf.
constexpr int kLgPieceIters = kLgPiece / (kLgThreads * 8);
template <bool BF16>
__device__ __forceinline__ void load_piece(const void* z, size_t base, int lo, int hi, int tid, float inv_temp,
                                           float (&y)[kLgPieceIters][8]) {
    if (BF16) {
        uint4 raw[kLgPieceIters];
#pragma unroll
        for (int it = 0; it < kLgPieceIters; ++it) {
            const int i = lo + (it * kLgThreads + tid) * 8;
            raw[it] = make_uint4(0xff80ff80u, 0xff80ff80u, 0xff80ff80u, 0xff80ff80u);  // bf16 -inf
            if (i < hi) raw[it] = *reinterpret_cast<const uint4*>(static_cast<const unsigned short*>(z) + base + i);
        }
#pragma unroll
        for (int it = 0; it < kLgPieceIters; ++it) {
            const unsigned w[4] = {raw[it].x, raw[it].y, raw[it].z, raw[it].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                y[it][2 * e] = mul_rn(__uint_as_float(w[e] << 16), inv_temp);
                y[it][2 * e + 1] = mul_rn(__uint_as_float(w[e] & 0xffff0000u), inv_temp);
            }
        }
    } else {
        float4 raw[kLgPieceIters][2];
#pragma unroll
        for (int it = 0; it < kLgPieceIters; ++it) {
            const int i = lo + (it * kLgThreads + tid) * 8;
            raw[it][0] = raw[it][1] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            if (i < hi) {
                raw[it][0] = *reinterpret_cast<const float4*>(static_cast<const float*>(z) + base + i);
                raw[it][1] = *reinterpret_cast<const float4*>(static_cast<const float*>(z) + base + i + 4);
            }
        }
#pragma unroll
        for (int it = 0; it < kLgPieceIters; ++it) {
            const float v[8] = {raw[it][0].x, raw[it][0].y, raw[it][0].z, raw[it][0].w,
                                raw[it][1].x, raw[it][1].y, raw[it][1].z, raw[it][1].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) y[it][e] = mul_rn(v[e], inv_temp);
        }
    }
}

__device__ __forceinline__ u128 shfl_down_u128(u128 v, int d) {
    const unsigned long long lo = shfl_down_u64((unsigned long long)v, d);
    const unsigned long long hi = shfl_down_u64((unsigned long long)(v >> 64), d);
    return ((u128)hi << 64) | lo;
}
__device__ __forceinline__ u128 shfl_up_u128(u128 v, int d) {
    const unsigned long long lo = shfl_up_u64((unsigned long long)v, d);
    const unsigned long long hi = shfl_up_u64((unsigned long long)(v >> 64), d);
    return ((u128)hi << 64) | lo;
}

// sum over a 256-thread workgroup, result in every thread
__device__ __forceinline__ u128 block_sum_u128(u128 v, u128* sh /*[kLgWaves]*/) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += shfl_down_u128(v, d);
    const int tid = threadIdx.x;
    __syncthreads();
    if ((tid & (kWave - 1)) == 0) sh[tid / kWave] = v;
    __syncthreads();
    u128 s = 0;
#pragma unroll
    for (int w = 0; w < kLgWaves; ++w) s += sh[w];
    return s;
}
// exclusive prefix sum in thread order over a 256-thread workgroup
__device__ __forceinline__ u128 block_excl_scan_u128(u128 v, u128* sh /*[kLgWaves]*/) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave;
    u128 incl = v;
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const u128 o = shfl_up_u128(incl, d);
        if (lane >= d) incl += o;
    }
    __syncthreads();
    if (lane == kWave - 1) sh[w] = incl;
    __syncthreads();
    u128 base = 0;
#pragma unroll
    for (int i = 0; i < kLgWaves; ++i) base += (i < w) ? sh[i] : (u128)0;
    return base + incl - v;
}

// row index of target row (b, j) and of draft row (b, j) in the stats array
__device__ __forceinline__ int trow(int b, int j, int k) { return b * (k + 1) + j; }
__device__ __forceinline__ int drow(int B, int b, int j, int k) { return B * (k + 1) + b * k + j; }

// Row statistics in two sweeps over pieces of kLgPiece logits (grid: pieces per row x rows), so that a
// row is spread over many compute units: piece maxima first; then, with the row maximum known, the
// integer weight sums of the pieces.  The second sweep finds the logits in the L2 / memory-side cache.
template <bool BF16, bool VEC>
__global__ __launch_bounds__(kLgThreads) void lg_max_kernel(int B, int k, int V, int npieces, const void* __restrict__ zt,
                                                            const void* __restrict__ zd, float inv_temp,
                                                            float* __restrict__ pmax,
                                                            unsigned long long* __restrict__ rsum) {
    __shared__ float sh_m[kLgWaves];
    const int r = blockIdx.x / npieces, pc = blockIdx.x - r * npieces, tid = threadIdx.x;
    const int nt = B * (k + 1);
    const void* z = r < nt ? zt : zd;
    const size_t base = (size_t)(r < nt ? r : r - nt) * V;
    const int lo = pc * kLgPiece, hi = min(V, lo + kLgPiece);
    float m = -INFINITY;
    if (VEC) {
        float y[kLgPieceIters][8];
        load_piece<BF16>(z, base, lo, hi, tid, inv_temp, y);
#pragma unroll
        for (int it = 0; it < kLgPieceIters; ++it)
#pragma unroll
            for (int e = 0; e < 8; ++e) m = fmaxf(m, y[it][e]);
    } else {
        for (int i = lo + tid; i < hi; i += kLgThreads) m = fmaxf(m, load_y<BF16>(z, base + i, inv_temp));
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) m = fmaxf(m, __shfl_xor(m, d, kWave));
    if ((tid & (kWave - 1)) == 0) sh_m[tid / kWave] = m;
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int w = 1; w < kLgWaves; ++w) m = fmaxf(m, sh_m[w]);
        pmax[(size_t)r * npieces + pc] = m;
        if (pc == 0) rsum[r] = 0ull;  // lg_sum_kernel adds the pieces' sums into it
    }
}

// Row maximum from the per-piece maxima.  The piece values are read in
// blocks of 16 independent loads: a plain loop would wait for every load before issuing the next and
// spend one memory latency per piece.
__device__ __forceinline__ float row_max(const float* pmax, int row, int npieces) {
    float m = -INFINITY;
    const float* src = pmax + (size_t)row * npieces;
    for (int i0 = 0; i0 < npieces; i0 += 16) {
        float v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = src[min(i0 + e, npieces - 1)];  // repeats of the last piece do no harm
#pragma unroll
        for (int e = 0; e < 16; ++e) m = fmaxf(m, v[e]);
    }
    return m;
}
// final statistics of a row, as lg_sum_kernel leaves them
__device__ __forceinline__ RowStat row_stat(const float* rmax, const unsigned long long* rsum, int row) {
    RowStat st;
    st.S = rsum[row];
    st.pad = 0.f;
    st.m = rmax[row];
    return st;
}

template <bool BF16, bool VEC>
__global__ __launch_bounds__(kLgThreads) void lg_sum_kernel(int B, int k, int V, int npieces, const void* __restrict__ zt,
                                                            const void* __restrict__ zd, float inv_temp,
                                                            const float* __restrict__ pmax,
                                                            float* __restrict__ rmax,
                                                            unsigned long long* __restrict__ rsum) {
    __shared__ unsigned long long sh_s[kLgWaves];
    const int r = blockIdx.x / npieces, pc = blockIdx.x - r * npieces, tid = threadIdx.x;
    const int nt = B * (k + 1);
    const void* z = r < nt ? zt : zd;
    const size_t base = (size_t)(r < nt ? r : r - nt) * V;
    const int lo = pc * kLgPiece, hi = min(V, lo + kLgPiece);
    const float m = row_max(pmax, r, npieces);
    unsigned long long s = 0;
    if (VEC) {
        float y[kLgPieceIters][8];
        load_piece<BF16>(z, base, lo, hi, tid, inv_temp, y);
#pragma unroll
        for (int it = 0; it < kLgPieceIters; ++it)
#pragma unroll
            for (int e = 0; e < 8; e += 2)  // two weights (each at most 2^30) fit 32 bits together
                s += logit_weight(y[it][e], m) + logit_weight(y[it][e + 1], m);
    } else {
        for (int i = lo + tid; i < hi; i += kLgThreads) s += logit_weight(load_y<BF16>(z, base + i, inv_temp), m);
    }
    s = wave_sum_u64(s);
    if ((tid & (kWave - 1)) == 0) sh_s[tid / kWave] = s;
    __syncthreads();
    if (tid == 0) {
        unsigned long long tot = 0;
#pragma unroll
        for (int w = 0; w < kLgWaves; ++w) tot += sh_s[w];
        atomicAdd(&rsum[r], tot);  // integers: the order of the pieces cannot matter
        if (pc == 0) rmax[r] = m;   // the row maximum, for the launches that follow
    }
}

// accepted length of branch b; every thread of the 256-thread workgroup gets it
template <bool BF16>
__device__ __forceinline__ int lg_accepted_length(int B, int b, int k, int V, const void* zt, const void* zd,
                                                  float inv_temp, const int32_t* draft, const float* u,
                                                  const float* rmax, const unsigned long long* rsum, int* sh_first) {
    const int tid = threadIdx.x;
    bool rejected = false;
    if (tid < k) {
        int x = draft[(size_t)b * k + tid];
        x = x < 0 ? 0 : (x >= V ? V - 1 : x);
        const RowStat sp = row_stat(rmax, rsum, trow(b, tid, k));
        const RowStat sq = row_stat(rmax, rsum, drow(B, b, tid, k));
        const unsigned long long Ep = logit_weight(load_y<BF16>(zt, (size_t)trow(b, tid, k) * V + x, inv_temp), sp.m);
        const unsigned long long Eq = logit_weight(load_y<BF16>(zd, ((size_t)b * k + tid) * V + x, inv_temp), sq.m);
        const u128 U = (u128)(unsigned)(u[(size_t)b * (k + 1) + tid] * 16777216.0f);
        rejected = !(U * Eq * sp.S < ((u128)1 << 24) * Ep * sq.S);
    }
    const unsigned long long mask = __ballot(rejected);
    if ((tid & (kWave - 1)) == 0) sh_first[tid / kWave] = mask ? (tid + __ffsll((long long)mask) - 1) : k;
    __syncthreads();
    int n = k;
#pragma unroll
    for (int w = 0; w < kLgWaves; ++w) n = sh_first[w] < n ? sh_first[w] : n;
    return n;
}

// the 8 weights a thread owns in a chunk (tokens lo .. lo+7, clipped to V): residual or plain
template <bool BF16, bool VEC>
__device__ __forceinline__ void lg_weights8(const void* zt_row, const void* zd_row, int lo, int V, float inv_temp,
                                            bool residual, RowStat sp, RowStat sq, u128 (&W)[8],
                                            unsigned long long (&Ep)[8]) {
    float yp[8], yq[8];
    if (VEC && lo + 8 <= V) {
        load_y8<BF16>(zt_row, lo, inv_temp, yp);
        if (residual) load_y8<BF16>(zd_row, lo, inv_temp, yq);
    } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const bool in = lo + e < V;
            yp[e] = in ? load_y<BF16>(zt_row, lo + e, inv_temp) : -INFINITY;
            yq[e] = (in && residual) ? load_y<BF16>(zd_row, lo + e, inv_temp) : -INFINITY;
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const bool in = lo + e < V;
        Ep[e] = in ? logit_weight(yp[e], sp.m) : 0ull;
        if (residual) {
            const unsigned long long Eq = in ? logit_weight(yq[e], sq.m) : 0ull;
            const u128 a = (u128)Ep[e] * sq.S, c = (u128)Eq * sp.S;
            W[e] = a > c ? a - c : (u128)0;
        } else {
            W[e] = Ep[e];
        }
    }
}

constexpr int kLgSpinLimit = 1 << 18;  // polls of the collecting workgroup before it gives up (far beyond any real wait)

// one published word: 32 bits of a sum under the call's tag
__device__ __forceinline__ void lg_publish(unsigned long long* slot, unsigned part, unsigned tag) {
    __hip_atomic_store(slot, ((unsigned long long)tag << 32) | part, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long lg_peek(const unsigned long long* slot) {
    return __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <bool BF16, bool VEC>
__global__ __launch_bounds__(kLgThreads) void lg_scan_pick_kernel(int B, int k, int V, int nchunks, unsigned tag,
                                                                  const void* __restrict__ zt, const void* __restrict__ zd,
                                                                  float inv_temp, const int32_t* __restrict__ draft,
                                                                  const float* __restrict__ u,
                                                                  const float* __restrict__ rmax,
                                                                  const unsigned long long* __restrict__ rsum,
                                                                  int32_t* __restrict__ accept_len,
                                                                  unsigned long long* __restrict__ slots,  // [B][nchunks][6]
                                                                  int32_t* __restrict__ next_token,
                                                                  int32_t* __restrict__ priv_len) {
    __shared__ int sh_first[kLgWaves];
    __shared__ u128 sh_w[kLgWaves];
    __shared__ u128 sh_base;
    __shared__ int sh_chunk, sh_bad;
    __shared__ u128 sh_wsum[kLgMaxChunks];
    __shared__ unsigned long long sh_psum[kLgMaxChunks];
    const int b = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
    const int n = lg_accepted_length<BF16>(B, b, k, V, zt, zd, inv_temp, draft, u, rmax, rsum, sh_first);
    bool residual = n < k;
    const size_t es = BF16 ? 2 : 4;
    const void* zt_row = static_cast<const char*>(zt) + (size_t)trow(b, n, k) * V * es;
    const void* zd_row = residual ? static_cast<const char*>(zd) + ((size_t)b * k + n) * V * es : zt_row;
    const RowStat sp = row_stat(rmax, rsum, trow(b, n, k));
    const RowStat sq = residual ? row_stat(rmax, rsum, drow(B, b, n, k)) : sp;
    u128 W[8];
    unsigned long long Ep[8];
    lg_weights8<BF16, VEC>(zt_row, zd_row, c * kLgChunk + tid * 8, V, inv_temp, residual, sp, sq, W, Ep);
    u128 w = 0, e = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        w += W[i];
        e += Ep[i];
    }
    w = block_sum_u128(w, sh_w);
    e = block_sum_u128(e, sh_w);
    unsigned long long* mine = slots + ((size_t)b * nchunks + c) * 6;
    if (tid == 0) {
        lg_publish(mine + 0, (unsigned)w, tag);
        lg_publish(mine + 1, (unsigned)(w >> 32), tag);
        lg_publish(mine + 2, (unsigned)(w >> 64), tag);
        lg_publish(mine + 3, (unsigned)(w >> 96), tag);
        lg_publish(mine + 4, (unsigned)e, tag);
        lg_publish(mine + 5, (unsigned)(e >> 32), tag);   // the plain sum of a chunk is below 2^41
    }
    if (c != nchunks - 1) return;  // uniform over the workgroup

    // ---- the branch's last chunk collects: it waits only for workgroups dispatched before it ----
    if (tid == 0) {
        accept_len[b] = n;
        if (priv_len) priv_len[b] -= k - n;  // the rejected drafts leave the branch's KV cache
        sh_bad = 0;
    }
    __syncthreads();
    for (int j = tid; j < nchunks; j += kLgThreads) {
        unsigned long long* en = slots + ((size_t)b * nchunks + j) * 6;
        unsigned long long v[6];
        bool ok = false;
        for (int spin = 0; spin < kLgSpinLimit; ++spin) {
            ok = true;
#pragma unroll
            for (int i = 0; i < 6; ++i) {
                v[i] = lg_peek(en + i);
                ok = ok && (unsigned)(v[i] >> 32) == tag;
            }
            if (ok) break;
            __builtin_amdgcn_s_sleep(1);
        }
        if (!ok) sh_bad = 1;  // never seen in practice: the producers were dispatched first and wait for nothing
        sh_wsum[j] = (u128)(unsigned)v[0] | ((u128)(unsigned)v[1] << 32) | ((u128)(unsigned)v[2] << 64) | ((u128)(unsigned)v[3] << 96);
        sh_psum[j] = (unsigned long long)(unsigned)v[4] | ((unsigned long long)(unsigned)v[5] << 32);
#pragma unroll
        for (int i = 0; i < 6; ++i)  // consumed: cleared, so that a captured launch (same tag) can be replayed
            __hip_atomic_store(en + i, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    // kLgMaxChunks = 2 * kLgThreads: every thread owns two consecutive chunk sums
    const int c0 = tid * 2;
    u128 w0 = 0, w1 = 0;
    unsigned long long p0 = 0, p1 = 0;
    if (c0 < nchunks) {
        w0 = sh_wsum[c0];
        p0 = sh_psum[c0];
    }
    if (c0 + 1 < nchunks) {
        w1 = sh_wsum[c0 + 1];
        p1 = sh_psum[c0 + 1];
    }
    u128 Z = block_sum_u128(w0 + w1, sh_w);
    if (residual && Z == 0) {  // empty residual: sample the target row itself (uniform branch: n and Z are)
        residual = false;
        w0 = p0;
        w1 = p1;
        Z = block_sum_u128(w0 + w1, sh_w);
    }
    if (Z == 0 || sh_bad) {  // a row without any weight (all logits -inf, or +inf / NaN among them): no token; uniform
        if (tid == 0) next_token[b] = -1;
        return;
    }
    unsigned m24 = (unsigned)(u[(size_t)b * (k + 1) + k] * 16777216.0f);
    m24 = m24 > 16777215u ? 16777215u : m24;  // u must be < 1; keeps T < Z regardless
    const u128 T = ((u128)m24 * Z) >> 24;
    u128 excl = block_excl_scan_u128(w0 + w1, sh_w);
    if (excl <= T && T < excl + w0 + w1) {  // exactly one thread: T < Z and Z > 0
        const bool second = !(T < excl + w0);
        sh_chunk = c0 + (second ? 1 : 0);
        sh_base = second ? excl + w0 : excl;
    }
    __syncthreads();
    const int cc = sh_chunk;
    const u128 base = sh_base;
    const void* zd_row2 = residual ? zd_row : zt_row;
    const RowStat sq2 = residual ? sq : sp;
    const int lo = cc * kLgChunk + tid * 8;
    lg_weights8<BF16, VEC>(zt_row, zd_row2, lo, V, inv_temp, residual, sp, sq2, W, Ep);
    u128 local = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) local += W[i];
    const u128 run = base + block_excl_scan_u128(local, sh_w);
    if (run <= T && T < run + local) {
        int tok = lo;
#pragma unroll
        for (int i = 7; i >= 0; --i) {  // the first i whose inclusive prefix exceeds T
            u128 pre = run;
#pragma unroll
            for (int j = 0; j <= i; ++j) pre += W[j];
            if (pre > T) tok = lo + i;
        }
        next_token[b] = tok;
    }
}


struct LgLayout {
    size_t off_pmax, off_rmax, off_rsum, off_wsum, off_psum, total;
    int nchunks, npieces;
};
static inline LgLayout lg_layout(int B, int k, int V) {
    LgLayout l;
    l.nchunks = (V + kLgChunk - 1) / kLgChunk;
    l.npieces = (V + kLgPiece - 1) / kLgPiece;
    const size_t rows = (size_t)B * (2 * k + 1);
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    l.off_pmax = 0;
    l.off_rmax = up(rows * l.npieces * sizeof(float));
    l.off_rsum = l.off_rmax + up(rows * sizeof(float));
    l.off_wsum = l.off_rsum + up(rows * sizeof(unsigned long long));
    l.off_psum = l.off_wsum;  // one block of tagged words: 6 per (branch, chunk)
    l.total = l.off_wsum + up((size_t)B * l.nchunks * 6 * sizeof(unsigned long long));
    return l;
}
static inline bool lg_sizes_ok(int B, int k, int V) {
    if (!(B >= 1 && B <= 65535 && k >= 0 && k <= kLgMaxK && V >= 1 && V <= (1 << 20))) return false;
    // one workgroup per (piece of a row, row): the launch must fit one grid dimension
    const long long pieces = (V + kLgPiece - 1) / kLgPiece;
    return pieces * B * (2 * k + 1) <= 0x7fffffffLL;
}

template <bool BF16, bool VEC>
static int lg_launch(int B, int k, int V, const void* zt, const void* zd, float inv_temp, const int32_t* draft,
                     const float* u, int32_t* accept_len, int32_t* next_token, int32_t* priv_len, void* workspace,
                     hipStream_t s) {
    const LgLayout l = lg_layout(B, k, V);
    float* pmax = reinterpret_cast<float*>(static_cast<char*>(workspace) + l.off_pmax);
    float* rmax = reinterpret_cast<float*>(static_cast<char*>(workspace) + l.off_rmax);
    unsigned long long* rsum = reinterpret_cast<unsigned long long*>(static_cast<char*>(workspace) + l.off_rsum);
    u128* wsum = reinterpret_cast<u128*>(static_cast<char*>(workspace) + l.off_wsum);
    const dim3 sgrid((unsigned)((long long)l.npieces * B * (2 * k + 1)));  // (piece, row) pairs, row-major
    LOTTS_LAUNCH((lg_max_kernel<BF16, VEC>), sgrid, dim3(kLgThreads), s, B, k, V, l.npieces, zt, zd, inv_temp, pmax,
                 rsum);
    int rc = check_launch();
    if (rc != LOTTS_OK) return rc;
    LOTTS_LAUNCH((lg_sum_kernel<BF16, VEC>), sgrid, dim3(kLgThreads), s, B, k, V, l.npieces, zt, zd, inv_temp, pmax,
                 rmax, rsum);
    rc = check_launch();
    if (rc != LOTTS_OK) return rc;
    const unsigned tag = next_word_tag();
    LOTTS_LAUNCH((lg_scan_pick_kernel<BF16, VEC>), dim3(l.nchunks, B), dim3(kLgThreads), s, B, k, V, l.nchunks, tag, zt, zd,
                 inv_temp, draft, u, rmax, rsum, accept_len, reinterpret_cast<unsigned long long*>(wsum), next_token,
                 priv_len);
    return check_launch();
}

}  // namespace lotts

extern "C" size_t spec_accept_logits_workspace_bytes(int32_t B, int32_t k, int32_t V) {
    if (!lotts::lg_sizes_ok(B, k, V)) return 0;
    return lotts::lg_layout(B, k, V).total;
}

extern "C" int spec_accept_logits(int32_t B, int32_t k, int32_t V, const void* target_logits, const void* draft_logits,
                                  int32_t logit_dtype, float inv_temperature, const int32_t* draft, const float* u,
                                  int32_t* accept_len, int32_t* next_token, int32_t* priv_len, void* workspace,
                                  size_t workspace_bytes, void* stream) {
    using namespace lotts;
    if (!lg_sizes_ok(B, k, V)) return LOTTS_ERR_SHAPE;
    if (logit_dtype != LOTTS_F32 && logit_dtype != LOTTS_BF16) return LOTTS_ERR_DTYPE;
    if (!(inv_temperature > 0.0f) || inv_temperature > 3.0e38f) return LOTTS_ERR_SHAPE;
    if (!target_logits || !u || !accept_len || !next_token || !workspace) return LOTTS_ERR_NULL;
    if (k > 0 && (!draft_logits || !draft)) return LOTTS_ERR_NULL;
    if (workspace_bytes < spec_accept_logits_workspace_bytes(B, k, V)) return LOTTS_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 15) != 0) return LOTTS_ERR_SHAPE;
    const bool bf16 = logit_dtype == LOTTS_BF16;
    const uintptr_t es = bf16 ? 2 : 4;
    if (((uintptr_t)target_logits | (uintptr_t)draft_logits) & (es - 1)) return LOTTS_ERR_SHAPE;
    // 8-wide loads need every row start 16-byte (bf16) / 32-byte-run (fp32: two 16-byte loads) aligned
    const bool vec = (V % 8 == 0) && ((((uintptr_t)target_logits | (uintptr_t)draft_logits) & 15) == 0);
    hipStream_t s = (hipStream_t)stream;
    if (bf16)
        return vec ? lg_launch<true, true>(B, k, V, target_logits, draft_logits, inv_temperature, draft, u, accept_len,
                                           next_token, priv_len, workspace, s)
                   : lg_launch<true, false>(B, k, V, target_logits, draft_logits, inv_temperature, draft, u, accept_len,
                                            next_token, priv_len, workspace, s);
    return vec ? lg_launch<false, true>(B, k, V, target_logits, draft_logits, inv_temperature, draft, u, accept_len,
                                        next_token, priv_len, workspace, s)
               : lg_launch<false, false>(B, k, V, target_logits, draft_logits, inv_temperature, draft, u, accept_len,
                                         next_token, priv_len, workspace, s);
}
