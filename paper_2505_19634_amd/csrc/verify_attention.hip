// verify_attention: causal attention of the k + 1 new positions of every branch against the
// branch's KV cache, which sits behind a prompt prefix shared by all branches (paper
// Section 3.2: B branches of one question; Section 2: the target model verifies the drafts in
// one parallel forward; Section 3.1: the step is bound by loading the KV cache).
//
// bf16 path (MFMA, gfx950), normally ONE launch:
//   attn_kernel           one launch over "work items", one workgroup each: 4 wavefronts for up to 32
//       query rows, 8 for up to 64 (two groups of 4, one row tile each; wavefront w of either group
//       streams the same key tiles, so the two load half a tile each into a slab both read).  An item
//       is a share of the keys of one KV segment and a stack of up to 32*NQT query rows that all
//       read those keys:
//         - private item: the G*R rows (G = Hq/Hkv query heads x R = k+1 positions) of one branch
//           and KV head, against a share of that branch's private keys;
//         - prefix item ("stacked" plan): rows of SEVERAL branches stacked on the MFMA N dimension
//           against a share of the shared prefix, so a prefix tile is fetched once per row stack
//           instead of once per branch;
//         - "folded" plan (prefix short next to the private caches): there are no prefix items;
//           each private item first runs its share of the prefix keys for its own rows (served by
//           the L2 after the first touch, so HBM still sees the prefix once) and continues into
//           the private keys with the same running state -- no extra partial, no extra workgroups.
//       The 32-key tiles of a segment are dealt round-robin to all wavefronts working on it; a
//       wavefront streams its tiles with coalesced non-temporal 16-byte loads into registers one
//       tile ahead, staged through a wavefront-private LDS slab
//       (K read back row-wise as the MFMA A operand, V with the transposing LDS load), S^T = K Q^T
//       and O^T += V^T P^T on 32x32x16 bf16 MFMA, flash-style running (max, sum, O).  The 4 states
//       are combined through LDS after one barrier and the item's un-normalised partial goes to
//       the workspace.  Arrivals are counted per (KV head, branch) in a cell that carries the call's
//       tag (what an earlier call left there, complete or not, counts as zero arrivals);
//       the workgroup that delivers the last partial does the log-sum-exp merge of that branch's
//       rows, normalises, converts and stores O (and LSE).  Partials cross workgroups -- and XCDs,
//       each with its own L2 -- inside one launch, so they are written and read with 16-byte
//       buffer accesses that carry the device-scope cache policy (performed at the memory side of
//       the L2s); nothing is ever flushed or invalidated cache-wide.
//   attn_merge_kernel     second launch, only when a row has many partials (few branches or long
//       caches): one workgroup would merge them at one compute unit's bandwidth, so the merge is
//       spread over the chip instead.
// fp32 path: attn_f32_kernel, plain fp32 VALU arithmetic, one workgroup per output row; it
// exists for exactness checks on small fp32 problems, not for speed.
// Two entry points share all of this: verify_attention (the caller brings the workspace) and
// verify_attention_noalloc (arrival cells and partials in a static device array of this file).
#include <atomic>
#include <cmath>

#include "lotts_common.h"

namespace lotts {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

constexpr int kAttnThreads = 256;
constexpr int kAttnWaves = kAttnThreads / kWave;
constexpr int kTile = 32;      // keys per tile = M of one 32x32x16 MFMA
constexpr int kRowTile = 32;   // query rows per row tile = N of the MFMA
constexpr int kMaxSplit = 16;  // more key shares than this cost more in the merge than they gain in streaming

struct AttnPlan {
    int nqt;            // row tiles per item: 1 or 2
    int fold;           // 1: private items also run their share of the prefix (no prefix items)
    int n_rg_priv;      // row groups per (branch, KV head)
    int n_rg_pre;       // row groups per KV head over all branches' stacked rows (stacked plan)
    int nsplit_priv;    // key splits of a private segment
    int nsplit_pre;     // key splits of the prefix (stacked plan; 0 otherwise)
    int nslots;         // partials per output row
    int fused;          // 1: the last-arriving workgroup merges inside the attention launch
    int n_pre_items, n_priv_items;
};

struct AttnParams {
    const void *Q, *Kpre, *Vpre, *Kpriv, *Vpriv;
    const int32_t* priv_len;
    void* ws;                  // workspace base; everything below lives in it
    unsigned ws_bytes;
    unsigned off_o, off_ml;    // byte offsets: partial O [Hkv][B*GR][nslots][D] fp32,
                               //               partial (running max in log2 units, sum) [Hkv][B*GR][nslots][2] fp32
    unsigned long long* counters;  // [Hkv][B] arrival cells at the start of the workspace: (call tag << 16) | arrivals
    unsigned long long tag;        // this call's tag, shifted into place: larger than that of any earlier call
    void* O;
    float* lse;
    int B, k, R, Hq, Hkv, G, GR, D, P, Lmax;
    unsigned g_magic;  // ceil(2^32 / G): x / G == umulhi(x, g_magic) for x * G < 2^32
    float scale_log2;  // scale * log2(e)
    long long q_stride_b, q_stride_r, q_stride_h;
    long long kpre_stride_h, kpre_stride_t;
    long long kpriv_stride_b, kpriv_stride_h, kpriv_stride_t;
    long long o_stride_b, o_stride_r, o_stride_h;
    AttnPlan plan;
};

static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Launch plan.  Depends on the descriptor only (never on device data), so the workspace query
// and the launch agree.  The HBM stream runs best with one streaming workgroup per compute
// unit, so the private caches are cut into just enough key shares to give every CU one item.
static inline AttnPlan plan_attention(const lotts_attn_desc& d) {
    AttnPlan pl;
    const int GR = (d.Hq / d.Hkv) * (d.k + 1);
    pl.nqt = GR > kRowTile ? 2 : 1;
    const int rows_per_item = kRowTile * pl.nqt;
    pl.n_rg_priv = ceil_div(GR, rows_per_item);
    pl.n_rg_pre = ceil_div(d.B * GR, rows_per_item);
    const int tiles_priv = ceil_div(d.Lmax, kTile);
    const long long base = (long long)d.B * d.Hkv * pl.n_rg_priv;
    long long want = (kNumCU + base - 1) / base;
    int max_split = tiles_priv / kAttnWaves;  // at least one tile per wavefront
    if (max_split > kMaxSplit) max_split = kMaxSplit;
    if (max_split < 1) max_split = 1;
    pl.nsplit_priv = (int)(want < 1 ? 1 : (want > max_split ? max_split : want));
    // A prefix that is short next to the private caches is folded into the private items.
    pl.fold = (d.P > 0 && (long long)d.P * 4 <= d.Lmax) ? 1 : 0;
    if (d.P > 0 && !pl.fold) {
        const int tiles_pre = ceil_div(d.P, kTile);
        const int tiles_per_item = ceil_div(tiles_priv, pl.nsplit_priv);
        int s = (tiles_pre + tiles_per_item / 2) / tiles_per_item;
        int cap = tiles_pre / kAttnWaves;
        if (cap > kMaxSplit) cap = kMaxSplit;
        if (s > cap) s = cap;
        pl.nsplit_pre = s < 1 ? 1 : s;
    } else {
        pl.nsplit_pre = 0;
    }
    pl.nslots = pl.nsplit_pre + pl.nsplit_priv;
    // The in-launch merge of a (KV head, branch) is done by ONE workgroup, at one CU's share of the
    // bandwidth: worth it only while that is a few tens of KB; beyond, a separate launch spreads the
    // merge over the whole chip.
    pl.fused = ((long long)pl.nslots * GR * d.D * 4 <= 48 * 1024) ? 1 : 0;
    pl.n_pre_items = d.Hkv * pl.n_rg_pre * pl.nsplit_pre;
    pl.n_priv_items = d.B * d.Hkv * pl.n_rg_priv * pl.nsplit_priv;
    return pl;
}

static inline size_t part_o_elems(const lotts_attn_desc& d, const AttnPlan& pl) {
    return (size_t)d.Hkv * d.B * (d.Hq / d.Hkv) * (d.k + 1) * pl.nslots * d.D;
}
static inline size_t part_ml_elems(const lotts_attn_desc& d, const AttnPlan& pl) {
    return (size_t)d.Hkv * d.B * (d.Hq / d.Hkv) * (d.k + 1) * pl.nslots * 2;
}

// Workspace: [arrival cells][partial O][partial (max, sum)], each part 256-byte aligned.  The
// cell block has the same place and size for every geometry, so a buffer stays usable when the
// geometry changes: partials of one call never land where another counts.
//
// An arrival cell holds (tag << 16) | arrivals.  Every call draws a tag larger than all earlier ones
// of this process; an arriving workgroup first raises the cell to (tag, 0) with an atomic maximum,
// then adds one.  A cell left at zero (a fresh zero-filled buffer, or the reset the last arriver
// does) and a cell left behind by an earlier call that never completed both start the new call
// at zero arrivals, so no call can poison the buffer for the next one.
constexpr int kMaxCounters = 16384;
constexpr int kTagShift = 16;            // arrivals per cell < 2^16, checked on the host
static std::atomic<unsigned long long> g_call_tag{0};
static inline size_t workspace_layout(const lotts_attn_desc& d, const AttnPlan& pl, size_t* off_o, size_t* off_ml) {
    size_t bytes = (size_t)kMaxCounters * sizeof(unsigned long long);
    if (off_o) *off_o = bytes;
    bytes += part_o_elems(d, pl) * sizeof(float);
    bytes = (bytes + 255) & ~(size_t)255;
    if (off_ml) *off_ml = bytes;
    bytes += part_ml_elems(d, pl) * sizeof(float);
    return (bytes + 255) & ~(size_t)255;
}

// 16- and 8-byte accesses to the workspace, with the device-scope cache policy (sc0 sc1) when the
// data crosses workgroups inside one launch, plain otherwise.
constexpr int kDevScope = 17;
__device__ __forceinline__ __amdgpu_buffer_rsrc_t ws_rsrc(const AttnParams& prm) {
    return __builtin_amdgcn_make_buffer_rsrc(prm.ws, 0, (int)prm.ws_bytes, 0x00020000);
}
template <bool DEV>
__device__ __forceinline__ void ws_store4(__amdgpu_buffer_rsrc_t r, unsigned byte_off, float4 v) {
    u32x4 u;
    u[0] = __float_as_uint(v.x); u[1] = __float_as_uint(v.y); u[2] = __float_as_uint(v.z); u[3] = __float_as_uint(v.w);
    __builtin_amdgcn_raw_buffer_store_b128(u, r, (int)byte_off, 0, DEV ? kDevScope : 0);
}
template <bool DEV>
__device__ __forceinline__ void ws_store2(__amdgpu_buffer_rsrc_t r, unsigned byte_off, float2 v) {
    u32x2 u;
    u[0] = __float_as_uint(v.x); u[1] = __float_as_uint(v.y);
    __builtin_amdgcn_raw_buffer_store_b64(u, r, (int)byte_off, 0, DEV ? kDevScope : 0);
}
template <bool DEV>
__device__ __forceinline__ float4 ws_load4(__amdgpu_buffer_rsrc_t r, unsigned byte_off) {
    const u32x4 u = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, DEV ? kDevScope : 0);
    return make_float4(__uint_as_float(u[0]), __uint_as_float(u[1]), __uint_as_float(u[2]), __uint_as_float(u[3]));
}
template <bool DEV>
__device__ __forceinline__ float2 ws_load2(__amdgpu_buffer_rsrc_t r, unsigned byte_off) {
    const u32x2 u = __builtin_amdgcn_raw_buffer_load_b64(r, (int)byte_off, 0, DEV ? kDevScope : 0);
    return make_float2(__uint_as_float(u[0]), __uint_as_float(u[1]));
}

// ---------------------------------------------------------------------------------------------
// Merge of the partials of the G*R output rows of one (KV head, branch), run by the workgroup that
// delivered the last of them:  O = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s, slots in index
// order whoever merges.  4 floats per output quad; a thread takes EU quads (256 apart) and CH
// slots at a time, so that EU * CH sixteen-byte loads are in flight together.  DEV selects
// device-scope loads (merge inside the attention launch, partials come from the memory side of the
// L2s) or plain loads (separate merge launch).  With OWN the merging workgroup's own partial (slot
// own_slot) is taken from its registers -- quad q of thread tid is quad tid + 256 q of the branch
// -- instead of being read back.
// ---------------------------------------------------------------------------------------------
template <int D, bool DEV, int EU, int CH, bool OWN>
__device__ __forceinline__ void merge_branch(const AttnParams& prm, __amdgpu_buffer_rsrc_t rs, int kvh, int b, int tid,
                                             int e_begin, int e_end, int own_slot, const float4 (&own_o)[EU],
                                             const float2 (&own_ml)[EU]) {
    constexpr int F4 = D / 4;
    const int ns = prm.plan.nslots;
    const int n_e = e_end < prm.GR * F4 ? e_end : prm.GR * F4;  // output quads [e_begin, e_end) of this (KV head, branch)
    for (int e0 = e_begin + tid; e0 < n_e; e0 += EU * kAttnThreads) {
        int rl[EU], c4[EU];
        unsigned base[EU];
        bool ok[EU];
        float M[EU], Lsum[EU];
        float4 o[EU];
#pragma unroll
        for (int q = 0; q < EU; ++q) {
            const int e = e0 + q * kAttnThreads;
            ok[q] = e < n_e;
            const int ec = ok[q] ? e : e0;
            rl[q] = ec / F4;
            c4[q] = ec - rl[q] * F4;
            base[q] = ((unsigned)kvh * prm.B * prm.GR + (unsigned)b * prm.GR + rl[q]) * ns;
            M[q] = -INFINITY;
            Lsum[q] = 0.f;
            o[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        for (int s0 = 0; s0 < ns; s0 += CH) {
            float2 mv[EU][CH];
            float4 pv[EU][CH];
#pragma unroll
            for (int q = 0; q < EU; ++q)
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    if (OWN && q * kAttnThreads >= n_e) continue;  // no thread has this quad (uniform)
                    const bool mine = OWN && s0 + j == own_slot;
                    const bool in = s0 + j < ns && !mine;
                    mv[q][j] = in ? ws_load2<DEV>(rs, prm.off_ml + (base[q] + s0 + j) * 8u) : make_float2(-INFINITY, 0.f);
                    pv[q][j] = in ? ws_load4<DEV>(rs, prm.off_o + ((base[q] + s0 + j) * D + c4[q] * 4) * 4u)
                                  : make_float4(0.f, 0.f, 0.f, 0.f);
                    if (mine) {
                        mv[q][j] = own_ml[q];
                        pv[q][j] = own_o[q];
                    }
                }
#pragma unroll
            for (int q = 0; q < EU; ++q) {
                if (OWN && q * kAttnThreads >= n_e) continue;
                float Mn = M[q];
#pragma unroll
                for (int j = 0; j < CH; ++j) Mn = fmaxf(Mn, mv[q][j].x);
                const float Mu = (Mn == -INFINITY) ? 0.f : Mn;
                const float a = __builtin_amdgcn_exp2f(M[q] - Mu);
                Lsum[q] *= a;
                o[q].x *= a; o[q].y *= a; o[q].z *= a; o[q].w *= a;
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    const float w = __builtin_amdgcn_exp2f(mv[q][j].x - Mu);
                    Lsum[q] += mv[q][j].y * w;
                    o[q].x += pv[q][j].x * w; o[q].y += pv[q][j].y * w;
                    o[q].z += pv[q][j].z * w; o[q].w += pv[q][j].w * w;
                }
                M[q] = Mn;
            }
        }
#pragma unroll
        for (int q = 0; q < EU; ++q) {
            if (!ok[q]) continue;
            const int r = prm.G == 1 ? rl[q] : (int)__umulhi((unsigned)rl[q], prm.g_magic), hg = rl[q] - r * prm.G;
            const int h = kvh * prm.G + hg;
            const float inv = 1.0f / Lsum[q];  // a row always sees itself: Lsum > 0
            __bf16* op = (__bf16*)prm.O + (long long)b * prm.o_stride_b + (long long)r * prm.o_stride_r +
                         (long long)h * prm.o_stride_h + c4[q] * 4;
            bf16x4 ov;
            ov[0] = (__bf16)(o[q].x * inv);
            ov[1] = (__bf16)(o[q].y * inv);
            ov[2] = (__bf16)(o[q].z * inv);
            ov[3] = (__bf16)(o[q].w * inv);
            *reinterpret_cast<bf16x4*>(op) = ov;
            if (prm.lse && c4[q] == 0)
                prm.lse[((long long)b * prm.R + r) * prm.Hq + h] = (M[q] + log2f(Lsum[q])) * 0.69314718055994530942f;
        }
    }
}
// the general form: every slot is read from the workspace, two quads and eight slots per round
template <int D, bool DEV>
__device__ __forceinline__ void merge_branch(const AttnParams& prm, __amdgpu_buffer_rsrc_t rs, int kvh, int b, int tid,
                                             int e_begin, int e_end) {
    const float4 no_o[2] = {};
    const float2 no_ml[2] = {};
    merge_branch<D, DEV, 2, 8, false>(prm, rs, kvh, b, tid, e_begin, e_end, -1, no_o, no_ml);
}

__device__ __forceinline__ bf16x8 load_bf16x8(const __bf16* ptr) {
    return *reinterpret_cast<const bf16x8*>(ptr);
}

// One run of keys a wavefront streams: tiles of 32 keys starting at `lo`, `step` keys apart,
// keys at or beyond `hi` do not belong to it.
struct KeyRun {
    const __bf16 *K, *V;
    long long stride_t;
    int lo, hi, step, ntiles;
};

// ---------------------------------------------------------------------------------------------
// bf16 partial attention
// ---------------------------------------------------------------------------------------------
template <int D, int NQT, int GROUPS>
__global__ __launch_bounds__(kAttnThreads * GROUPS, (NQT > 1 ? 1 : 2)) void attn_kernel(const AttnParams prm) {
    // GROUPS = 2: eight wavefronts, two per SIMD.  The second group of four takes the second row tile; wavefront w of
    // either group streams the same key tiles, so the two share them: each loads half of a tile into a slab both
    // read (two slabs per pair, taking turns; the pair meets once per tile at a counter in LDS, the four pairs stay
    // independent of each other).
    static_assert(GROUPS == 1 || (GROUPS == 2 && NQT == 2), "two groups split two row tiles");
    constexpr int TW = NQT / GROUPS;       // row tiles per wavefront
    constexpr int KS = D / 16;             // MFMA k-steps of the QK^T contraction
    constexpr int DB = D / 32;             // 32-wide blocks of the head dimension
    constexpr int KSTRIDE = D * 2 + 16;    // bytes per key row of the K slab (pad: conflict-free 16-byte row reads)
    constexpr int VSTRIDE = D * 2 + 64;    // bytes per key row of the V slab (pad: conflict-free transposing reads)
    constexpr int KSLAB = kTile * KSTRIDE, VSLAB = kTile * VSTRIDE;
    constexpr int SLAB = KSLAB + VSLAB;    // bytes of LDS per wavefront while streaming
    constexpr int OSTRIDE = D + 4;         // floats per row of a wavefront's merge buffer
    constexpr int OBUF = kRowTile * OSTRIDE * 4;
    static_assert(OBUF <= SLAB, "the merge buffer reuses the wavefront's slab");
    __shared__ __attribute__((aligned(16))) unsigned char lds[kAttnWaves * GROUPS * SLAB];
    __shared__ float sh_m[kAttnWaves * GROUPS][kRowTile];
    __shared__ float sh_l[kAttnWaves * GROUPS][kRowTile];
    __shared__ int sh_pair[kAttnWaves];  // GROUPS = 2: half tiles stored by the pair of wavefronts w and w + 4

    const int tid = threadIdx.x, wave_all = tid / kWave, lane = tid & (kWave - 1);
    const int grp = GROUPS == 1 ? 0 : wave_all / kAttnWaves;         // which row tile(s) this wavefront works on
    const int wave = GROUPS == 1 ? wave_all : wave_all % kAttnWaves;  // which of the item's four runs of key tiles it streams
    const int ln = lane & 31;   // MFMA column (query row) / A row (key or d) owned by this lane
    const int hh = lane >> 5;   // which half of each 16-wide k block this lane holds
    const AttnPlan& pl = prm.plan;
    const int GR = prm.GR;

    // ---- decode the work item: private items first (one per CU starts at once), prefix items after ----
    // Order matters for latency: whatever does not depend on priv_len[b] (the prefix share, the Q
    // rows) is requested before that value is first used.
    int id = blockIdx.x;
    const bool is_private = id < pl.n_priv_items;
    int kvh, split, nsplit, rho0, rho_end, slot, b_item = 0;
    KeyRun run[2];   // run[0]: folded prefix share (may be empty), run[1]: the item's own segment
    run[0].ntiles = 0;
    if (is_private) {
        kvh = id % prm.Hkv;
        int rest = id / prm.Hkv;
        split = rest % pl.nsplit_priv;
        rest /= pl.nsplit_priv;
        const int rg = rest % pl.n_rg_priv;
        b_item = rest / pl.n_rg_priv;
        nsplit = pl.nsplit_priv;
        rho0 = b_item * GR + rg * kRowTile * NQT;
        rho_end = min((b_item + 1) * GR, rho0 + kRowTile * NQT);
        slot = pl.nsplit_pre + split;
    } else {
        id -= pl.n_priv_items;
        kvh = id % prm.Hkv;
        int rest = id / prm.Hkv;
        split = rest % pl.nsplit_pre;
        const int rg = rest / pl.nsplit_pre;
        nsplit = pl.nsplit_pre;
        rho0 = rg * kRowTile * NQT;
        rho_end = min(prm.B * GR, rho0 + kRowTile * NQT);
        slot = split;
    }
    const int L_raw = is_private ? prm.priv_len[b_item] : 0;  // requested here, first used further down
    // The 32-key tiles of a segment are dealt round-robin to all wavefronts working on it (the 4
    // wavefronts of each of its nsplit items): every wavefront streams the same number of tiles to
    // within one whatever the segment's length, and at any moment the wavefronts of a segment read
    // neighbouring tiles, which spreads each item's traffic over the memory channels.
    const int wave_of_seg = split * kAttnWaves + wave, waves_of_seg = nsplit * kAttnWaves;
    if (is_private && pl.fold) {
        run[0].K = (const __bf16*)prm.Kpre + (long long)kvh * prm.kpre_stride_h;
        run[0].V = (const __bf16*)prm.Vpre + (long long)kvh * prm.kpre_stride_h;
        run[0].stride_t = prm.kpre_stride_t;
        run[0].lo = wave_of_seg * kTile;
        run[0].hi = prm.P;
        run[0].step = waves_of_seg * kTile;
        run[0].ntiles = run[0].lo < run[0].hi ? (run[0].hi - run[0].lo + run[0].step - 1) / run[0].step : 0;
    }
    const int n_fold = run[0].ntiles;

    unsigned char* kslab = lds + wave * SLAB;  // GROUPS = 2: re-pointed every tile
    unsigned char* vslab = kslab + KSLAB;
    // Tile staging: every load instruction of the wavefront covers RPI whole key rows (16 bytes per
    // lane, consecutive lanes consecutive addresses), the same pattern for K and V.
    constexpr int LPR = D / 8;             // lanes per key row
    constexpr int RPI = kWave / LPR;       // key rows per load instruction
    constexpr int NVL = kTile / RPI;       // load instructions per tile and operand
    const int v_row = lane / LPR, v_chunk = lane % LPR;
    // transposing-read address of this lane inside the V slab: 16-lane blocks cover 4 keys x 16 d
    const int blk = lane >> 4, i16 = lane & 15;
    const int tr_off = ((blk >> 1) * 4 + (i16 >> 2)) * VSTRIDE + ((blk & 1) * 16 + (i16 & 3) * 4) * 2;

    // The next tile is fetched into registers while the current one is being consumed from LDS.
    // K and V are read exactly once, so the loads carry the non-temporal hint.
    constexpr int NLD = NVL / GROUPS;      // load instructions per tile and operand issued by this wavefront
    u32x4 kst[NLD], vst[NLD];
    auto fetch = [&](int it) {
        const KeyRun& r = run[it < n_fold ? 0 : 1];
        const int kb_ = r.lo + (it < n_fold ? it : it - n_fold) * r.step;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            int key = kb_ + (i * GROUPS + grp) * RPI + v_row;
            key = key < r.hi ? key : r.hi - 1;  // a ragged last tile re-reads its last row; masked below
            const long long off = (long long)key * r.stride_t + v_chunk * 8;
            kst[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(r.K + off));
            vst[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(r.V + off));
        }
    };
    if (n_fold > 0) fetch(0);

    // ---- Q fragments (B operand of S^T = K Q^T: lane = query row ln, 8 contiguous d) ----
    bf16x8 qf[TW][KS];
    int q_r[TW];  // position (0..k) of this lane's query row
#pragma unroll
    for (int t = 0; t < TW; ++t) {
        const int rho = rho0 + (grp * TW + t) * kRowTile + ln;
        const bool valid = rho < rho_end;
        const int rc = valid ? rho : rho0;
        const int b = rc / GR, rl = rc - b * GR;
        const int r = rl / prm.G, hg = rl - r * prm.G;
        q_r[t] = r;
        const __bf16* qp = (const __bf16*)prm.Q + (long long)b * prm.q_stride_b + (long long)r * prm.q_stride_r +
                           (long long)(kvh * prm.G + hg) * prm.q_stride_h;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            bf16x8 v = load_bf16x8(qp + (2 * s + hh) * 8);
            if (!valid) {
#pragma unroll
                for (int j = 0; j < 8; ++j) v[j] = (__bf16)0.0f;
            }
            qf[t][s] = v;
        }
    }

    // ---- the item's own segment ----
    int seg_len, causal_base;
    if (is_private) {
        const int L = L_raw < prm.R ? prm.R : (L_raw > prm.Lmax ? prm.Lmax : L_raw);
        seg_len = L;
        causal_base = L - prm.k;  // row at position r sees private keys [0, L - k + r)
        const long long off = (long long)b_item * prm.kpriv_stride_b + (long long)kvh * prm.kpriv_stride_h;
        run[1].K = (const __bf16*)prm.Kpriv + off;
        run[1].V = (const __bf16*)prm.Vpriv + off;
        run[1].stride_t = prm.kpriv_stride_t;
    } else {
        seg_len = prm.P;
        causal_base = prm.P;  // every row sees the whole prefix
        run[1].K = (const __bf16*)prm.Kpre + (long long)kvh * prm.kpre_stride_h;
        run[1].V = (const __bf16*)prm.Vpre + (long long)kvh * prm.kpre_stride_h;
        run[1].stride_t = prm.kpre_stride_t;
    }
    // The dealing goes on where the folded prefix tiles stopped: prefix and private tiles form one
    // sequence, so a wavefront that got one prefix tile more gets one private tile less.
    int first_wave = 0;
    if (is_private && pl.fold) first_wave = ((prm.P + kTile - 1) / kTile) % waves_of_seg;
    run[1].lo = ((wave_of_seg - first_wave + waves_of_seg) % waves_of_seg) * kTile;
    run[1].hi = seg_len;
    run[1].step = waves_of_seg * kTile;
    run[1].ntiles = run[1].lo < seg_len ? (seg_len - run[1].lo + run[1].step - 1) / run[1].step : 0;
    const int n_tiles = n_fold + run[1].ntiles;
    if (n_fold == 0 && n_tiles > 0) fetch(0);
    int lim[TW];  // keys of this wavefront's own run visible to this lane's query row
#pragma unroll
    for (int t = 0; t < TW; ++t) lim[t] = min(is_private ? causal_base + q_r[t] : causal_base, run[1].hi);

    // ---- running state ----
    f32x16 oacc[TW][DB];
    float m_run[TW], l_run[TW];
#pragma unroll
    for (int t = 0; t < TW; ++t) {
        m_run[t] = -INFINITY;
        l_run[t] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[t][db][i] = 0.f;
    }

    if (GROUPS > 1) {  // the two wavefronts of a pair count their half tiles here
        if (tid < kAttnWaves) sh_pair[tid] = 0;
        __syncthreads();
    }
    for (int it = 0; it < n_tiles; ++it) {
        const bool folded = it < n_fold;
        const int kbase = folded ? run[0].lo + it * run[0].step : run[1].lo + (it - n_fold) * run[1].step;
        if (GROUPS > 1) {
            kslab = lds + ((it & 1) * kAttnWaves + wave) * SLAB;
            vslab = kslab + KSLAB;
        }
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            *reinterpret_cast<u32x4*>(kslab + ((i * GROUPS + grp) * RPI + v_row) * KSTRIDE + v_chunk * 16) = kst[i];
            *reinterpret_cast<u32x4*>(vslab + ((i * GROUPS + grp) * RPI + v_row) * VSTRIDE + v_chunk * 16) = vst[i];
        }
        if (GROUPS > 1) {
            // both halves written: the pair's counter stands at 2 * (it + 1).  Whoever gets past this has also left
            // the tile before behind (it counted this tile only after that), so the other slab is free.
            if (lane == 0) __hip_atomic_fetch_add(&sh_pair[wave], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
            for (int spin = 0; spin < (1 << 20); ++spin) {  // the partner runs the same tiles: the wait ends; bounded all the same
                if (__hip_atomic_load(&sh_pair[wave], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) >= 2 * (it + 1)) break;
                __builtin_amdgcn_s_sleep(1);
            }
        }
        if (it + 1 < n_tiles) fetch(it + 1);
        // K fragments (A operand of S^T = K Q^T: lane = key row ln, 8 contiguous d)
        bf16x8 kf[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s)
            kf[s] = *reinterpret_cast<const bf16x8*>(kslab + ln * KSTRIDE + (2 * s + hh) * 16);

        bf16x8 pf[TW][2];
#pragma unroll
        for (int t = 0; t < TW; ++t) {
            // S^T[key][query] = sum_d K[key][d] Q[query][d]
            f32x16 acc;
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
            for (int s = 0; s < KS; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[t][s], acc, 0, 0, 0);
            // register i of this lane is key kbase + (i/4)*8 + hh*4 + i%4 for query row ln;
            // every row sees all of a prefix share, the causal limit applies to the own run only
            const int vis = (folded ? run[0].hi : lim[t]) - kbase - hh * 4;  // key offsets below this are visible
            float mx = -INFINITY;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int koff = (i >> 2) * 8 + (i & 3);
                float sc = acc[i] * prm.scale_log2;
                sc = koff < vis ? sc : -INFINITY;
                acc[i] = sc;
                mx = fmaxf(mx, sc);
            }
            mx = fmaxf(mx, shfl_xor_f(mx, 32));
            const float m_new = fmaxf(m_run[t], mx);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run[t] - m_use);
            float psum = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float pv = __builtin_amdgcn_exp2f(acc[i] - m_use);
                psum += pv;
                pf[t][i >> 3][i & 7] = (__bf16)pv;
            }
            l_run[t] = l_run[t] * alpha + psum;
            m_run[t] = m_new;
            // Rescaling the accumulators is the largest block of vector work of a tile, and once a few hundred keys have
            // gone by a tile rarely raises any row's maximum: alpha is exactly 1 for every lane then and the whole
            // wavefront skips it (multiplying by 1 changes nothing, so the result is the same bit for bit).
            if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int i = 0; i < 16; ++i) oacc[t][db][i] *= alpha;
            }
        }
        // O^T[d][query] += sum_key V[key][d] P^T[key][query]; V^T fragments by transposing LDS reads
#pragma unroll
        for (int db = 0; db < DB; ++db) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const unsigned char* ap = vslab + tr_off + (kb * 16) * VSTRIDE + db * 64;
                const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) short4v*)(ap));
                const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) short4v*)(ap + 8 * VSTRIDE));
                union {
                    short4v s[2];
                    bf16x8 v;
                } vf;
                vf.s[0] = lo;
                vf.s[1] = hi;
#pragma unroll
                for (int t = 0; t < TW; ++t)
                    oacc[t][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf[t][kb], oacc[t][db], 0, 0, 0);
            }
        }
    }

    // ---- combine the 4 wavefronts' states of a row tile (fixed order) and store the item's partial ----
    // Each wavefront parks its raw state in LDS (its slab is free now); after one barrier the 256 threads
    // of a group of four wavefronts form sum_w 2^(m_w - m) O_w over their group and write the valid rows out,
    // coalesced (two groups: both row tiles at the same time).  A thread owns QPT output quads of a row
    // tile -- quad t + 256 q, t its number within the group: the same column of rows RSTEP apart -- and
    // reads everything it needs for all of them before it uses any of it.
    constexpr int F4 = D / 4;
    constexpr int QPT = kRowTile * F4 / kAttnThreads;  // 4 (D = 128) or 2 (D = 64)
    constexpr int RSTEP = kAttnThreads / F4;
    if (GROUPS > 1) __syncthreads();  // nobody reads a key tile any more: the slabs become merge buffers
    float* obuf = reinterpret_cast<float*>(lds + wave_all * SLAB);
    const __amdgpu_buffer_rsrc_t rs = ws_rsrc(prm);
    const int tig = tid % kAttnThreads;  // thread within its group of four wavefronts
    const int c4 = tig % F4, row0 = tig / F4;
    float4 own_o[QPT];    // the last row tile's combined quads, kept for a merge by this workgroup
    float2 own_ml[QPT];
#pragma unroll
    for (int t = 0; t < TW; ++t) {
        if (t > 0) __syncthreads();  // the previous row tile has been read out
        const int tile = grp * TW + t;  // row tile of the item
        const float lsum = l_run[t] + shfl_xor_f(l_run[t], 32);
        if (hh == 0) {
            sh_m[wave_all][ln] = m_run[t];
            sh_l[wave_all][ln] = lsum;
        }
        const int nrows = min(kRowTile, rho_end - (rho0 + tile * kRowTile));
        if (ln < nrows) {  // rows beyond the item's are never read back
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    *reinterpret_cast<float4*>(obuf + ln * OSTRIDE + db * 32 + q4 * 8 + hh * 4) =
                        make_float4(oacc[t][db][q4 * 4 + 0], oacc[t][db][q4 * 4 + 1], oacc[t][db][q4 * 4 + 2],
                                    oacc[t][db][q4 * 4 + 3]);
        }
        __syncthreads();
        float mw[QPT][kAttnWaves], lw[QPT][kAttnWaves];
        float4 ov[QPT][kAttnWaves];
#pragma unroll
        for (int q = 0; q < QPT; ++q)
#pragma unroll
            for (int w = 0; w < kAttnWaves; ++w) {
                if (q * RSTEP >= nrows) continue;  // a whole group of rows beyond the item's (uniform)
                const int row = min(row0 + q * RSTEP, nrows - 1);
                mw[q][w] = sh_m[grp * kAttnWaves + w][row];
                lw[q][w] = sh_l[grp * kAttnWaves + w][row];
                ov[q][w] = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(lds + (grp * kAttnWaves + w) * SLAB) +
                                                            row * OSTRIDE + c4 * 4);
            }
#pragma unroll
        for (int q = 0; q < QPT; ++q) {
            if (q * RSTEP >= nrows) continue;
            const int row = row0 + q * RSTEP;
            float mg = -INFINITY;
#pragma unroll
            for (int w = 0; w < kAttnWaves; ++w) mg = fmaxf(mg, mw[q][w]);
            const float mg_use = (mg == -INFINITY) ? 0.f : mg;
            float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
            float lg = 0.f;
#pragma unroll
            for (int w = 0; w < kAttnWaves; ++w) {
                const float sc = __builtin_amdgcn_exp2f(mw[q][w] - mg_use);
                o.x += ov[q][w].x * sc;
                o.y += ov[q][w].y * sc;
                o.z += ov[q][w].z * sc;
                o.w += ov[q][w].w * sc;
                lg += lw[q][w] * sc;
            }
            own_o[q] = o;
            own_ml[q] = make_float2(mg, lg);
            if (row < nrows) {
                const unsigned rho = rho0 + tile * kRowTile + row;
                const unsigned pidx = ((unsigned)kvh * prm.B * GR + rho) * pl.nslots + slot;
                if (pl.fused) {
                    ws_store4<true>(rs, prm.off_o + (pidx * D + c4 * 4) * 4u, o);
                    if (c4 == 0) ws_store2<true>(rs, prm.off_ml + pidx * 8u, make_float2(mg, lg));
                } else {
                    ws_store4<false>(rs, prm.off_o + (pidx * D + c4 * 4) * 4u, o);
                    if (c4 == 0) ws_store2<false>(rs, prm.off_ml + pidx * 8u, make_float2(mg, lg));
                }
            }
        }
    }

    if (!pl.fused) return;  // a separate launch merges (many partials per row: one workgroup would be too slow)
    // ---- arrival: whoever completes the set of partials of a (KV head, branch) merges it ----
    // Every thread waits until its partial stores are acknowledged; then one thread per covered
    // branch counts the arrival in that branch's cell: raise it to (this call's tag, 0) if it holds
    // anything older, add one.  The two atomics go to one address from one thread, so they take
    // effect in program order.  The last arrival puts a zero back, which lets a captured launch
    // (same tag every time) be replayed.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    int* sh_last = reinterpret_cast<int*>(sh_l);  // free again; kAttnWaves * kRowTile >= rows of an item
    const int rows_per_item = kRowTile * NQT;
    const int b_first = rho0 / GR, b_last = (rho_end - 1) / GR;
    const int nb = b_last - b_first + 1;  // <= rows_per_item
    if (tid < nb) {
        const int b = b_first + tid;
        int expected = pl.n_rg_priv * pl.nsplit_priv;
        if (pl.nsplit_pre > 0) {
            const int rg_lo = (b * GR) / rows_per_item, rg_hi = ((b + 1) * GR - 1) / rows_per_item;
            expected += pl.nsplit_pre * (rg_hi - rg_lo + 1);
        }
        unsigned long long* cnt = prm.counters + kvh * prm.B + b;
        atomicMax(cnt, prm.tag);
        const unsigned long long seen = atomicAdd(cnt, 1ull);
        const int last = (seen == prm.tag + (unsigned long long)(expected - 1));
        if (last) atomicExch(cnt, 0ull);
        sh_last[tid] = last;
    }
    __syncthreads();
    // The common shape -- the item's rows are exactly one branch's rows and every partial of the branch
    // comes from an item like this one -- merges all of the thread's quads in one round of loads and
    // takes this workgroup's own partial from its registers; everything else goes the general way.
    if (NQT == 1 && is_private && pl.n_rg_priv == 1 && pl.nsplit_pre == 0) {
        if (sh_last[0]) merge_branch<D, true, QPT, 2, true>(prm, rs, kvh, b_item, tid, 0, 1 << 30, slot, own_o, own_ml);
    } else {
        if (GROUPS == 1 || tid < kAttnThreads)  // the merge is written for 256 threads
            for (int j = 0; j < nb; ++j)
                if (sh_last[j]) merge_branch<D, true>(prm, rs, kvh, b_first + j, tid, 0, 1 << 30);  // uniform over the workgroup
    }
    __builtin_amdgcn_s_waitcnt(0);
}

// ---------------------------------------------------------------------------------------------
// Separate merge launch, used when a row has many partials: grid (quads of a (KV head, branch) in
// blocks of 256, KV head x branch), one output quad per thread, so the whole chip shares the reads.
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kAttnThreads) void attn_merge_kernel(const AttnParams prm) {
    const int kvh = blockIdx.y % prm.Hkv, b = blockIdx.y / prm.Hkv;
    const int e_begin = blockIdx.x * kAttnThreads;
    merge_branch<D, false>(prm, ws_rsrc(prm), kvh, b, threadIdx.x, e_begin, e_begin + kAttnThreads);
}

// ---------------------------------------------------------------------------------------------
// fp32 path: one workgroup per output row, fp32 arithmetic throughout (no matrix cores).
// Wavefront w takes keys w, w+4, ...; lanes split the head dimension; flash-style running state
// per wavefront, merged through LDS.
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(kAttnThreads) void attn_f32_kernel(const AttnParams prm) {
    constexpr int EPL = D / kWave;  // head-dim elements per lane
    __shared__ float sh_acc[kAttnWaves][D];
    __shared__ float sh_ml[kAttnWaves][2];
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid & (kWave - 1);
    const long long row = blockIdx.x;
    const int h = (int)(row % prm.Hq);
    const long long br = row / prm.Hq;
    const int r = (int)(br % prm.R), b = (int)(br / prm.R);
    const int kvh = h / prm.G;
    int L = prm.priv_len[b];
    L = L < prm.R ? prm.R : (L > prm.Lmax ? prm.Lmax : L);
    const int n_priv = L - prm.k + r;
    const int n = prm.P + n_priv;
    const float scale = prm.scale_log2 * 0.69314718055994530942f;  // back to the natural-log scale
    const float* qp = (const float*)prm.Q + (long long)b * prm.q_stride_b + (long long)r * prm.q_stride_r +
                      (long long)h * prm.q_stride_h;
    float qv[EPL], acc[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        qv[e] = qp[lane + e * kWave];
        acc[e] = 0.f;
    }
    float m = -INFINITY, l = 0.f;
    for (int j = wave; j < n; j += kAttnWaves) {
        const float *kp, *vp;
        if (j < prm.P) {
            const long long off = (long long)kvh * prm.kpre_stride_h + (long long)j * prm.kpre_stride_t;
            kp = (const float*)prm.Kpre + off;
            vp = (const float*)prm.Vpre + off;
        } else {
            const long long off = (long long)b * prm.kpriv_stride_b + (long long)kvh * prm.kpriv_stride_h +
                                  (long long)(j - prm.P) * prm.kpriv_stride_t;
            kp = (const float*)prm.Kpriv + off;
            vp = (const float*)prm.Vpriv + off;
        }
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) s += qv[e] * kp[lane + e * kWave];
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) s += shfl_xor_f(s, d);
        s *= scale;
        const float m_new = fmaxf(m, s);
        const float alpha = expf(m - m_new);
        const float pv = expf(s - m_new);
        l = l * alpha + pv;
        m = m_new;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] = acc[e] * alpha + pv * vp[lane + e * kWave];
    }
    if (lane == 0) {
        sh_ml[wave][0] = m;
        sh_ml[wave][1] = l;
    }
#pragma unroll
    for (int e = 0; e < EPL; ++e) sh_acc[wave][lane + e * kWave] = acc[e];
    __syncthreads();
    if (tid < D) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) M = fmaxf(M, sh_ml[w][0]);
        float Lsum = 0.f, o = 0.f;
#pragma unroll
        for (int w = 0; w < kAttnWaves; ++w) {
            const float wgt = (sh_ml[w][0] == -INFINITY) ? 0.f : expf(sh_ml[w][0] - M);
            Lsum += sh_ml[w][1] * wgt;
            o += sh_acc[w][tid] * wgt;
        }
        float* op = (float*)prm.O + (long long)b * prm.o_stride_b + (long long)r * prm.o_stride_r +
                    (long long)h * prm.o_stride_h;
        op[tid] = o / Lsum;
        if (prm.lse && tid == 0) prm.lse[row] = M + logf(Lsum);
    }
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
static int fill_desc(const lotts_attn_desc* in, lotts_attn_desc* d) {
    if (!in) return LOTTS_ERR_NULL;
    *d = *in;
    if (d->dtype != LOTTS_F32 && d->dtype != LOTTS_BF16) return LOTTS_ERR_DTYPE;
    if (d->B < 1 || d->k < 0 || d->Hq < 1 || d->Hkv < 1 || d->Hq % d->Hkv != 0) return LOTTS_ERR_SHAPE;
    if (d->D != 64 && d->D != 128) return LOTTS_ERR_SHAPE;
    if (d->P < 0 || d->Lmax < d->k + 1) return LOTTS_ERR_SHAPE;
    if (!(d->scale >= 0.0f) || d->scale > 3.0e38f) return LOTTS_ERR_SHAPE;
    const long long R = d->k + 1, D = d->D;
    // 0 selects the dense layout
    if (!d->q_stride_h) d->q_stride_h = D;
    if (!d->q_stride_r) d->q_stride_r = (long long)d->Hq * D;
    if (!d->q_stride_b) d->q_stride_b = R * d->Hq * D;
    if (!d->o_stride_h) d->o_stride_h = D;
    if (!d->o_stride_r) d->o_stride_r = (long long)d->Hq * D;
    if (!d->o_stride_b) d->o_stride_b = R * d->Hq * D;
    if (!d->kpre_stride_t) d->kpre_stride_t = D;
    if (!d->kpre_stride_h) d->kpre_stride_h = (long long)d->P * D;
    if (!d->kpriv_stride_t) d->kpriv_stride_t = D;
    if (!d->kpriv_stride_h) d->kpriv_stride_h = (long long)d->Lmax * D;
    if (!d->kpriv_stride_b) d->kpriv_stride_b = (long long)d->Hkv * d->Lmax * D;
    const long long st[] = {d->q_stride_b, d->q_stride_r, d->q_stride_h, d->kpre_stride_h, d->kpre_stride_t,
                            d->kpriv_stride_b, d->kpriv_stride_h, d->kpriv_stride_t, d->o_stride_b, d->o_stride_r,
                            d->o_stride_h};
    for (long long s : st) {
        if (s < 0) return LOTTS_ERR_SHAPE;
        if (d->dtype == LOTTS_BF16 && (s % 8) != 0) return LOTTS_ERR_SHAPE;  // 16-byte vector loads
    }
    if (d->q_stride_h < D || d->o_stride_h < D || d->kpre_stride_t < D || d->kpriv_stride_t < D) return LOTTS_ERR_SHAPE;
    const long long rows = (long long)d->B * R * d->Hq;
    if (rows > 0x7fffffffLL / 8) return LOTTS_ERR_SHAPE;
    if ((long long)d->B * d->Hkv > kMaxCounters) return LOTTS_ERR_SHAPE;
    return LOTTS_OK;
}

// Bytes of workspace for a checked descriptor; 0 when the geometry cannot be served (partials are
// addressed with 32-bit byte offsets, arrivals per cell are counted in 16 bits).
static size_t workspace_need(const lotts_attn_desc& d) {
    if (d.dtype == LOTTS_F32) return 256;  // the fp32 path needs none; keep the pointer non-NULL
    const AttnPlan pl = plan_attention(d);
    const long long arrivals = (long long)pl.n_rg_priv * pl.nsplit_priv + (long long)pl.nsplit_pre * (pl.n_rg_priv + 1);
    if (arrivals >= (1 << kTagShift)) return 0;
    const size_t bytes = workspace_layout(d, pl, nullptr, nullptr);
    return bytes < 0x7fffffffULL ? bytes : 0;
}

// Everything after the argument checks that both entry points share: plan, parameters, launches.
// `workspace` holds at least workspace_need(d) bytes.
static int launch_attention(const lotts_attn_desc& d, const void* Q, const void* Kpre, const void* Vpre,
                            const void* Kpriv, const void* Vpriv, const int32_t* priv_len, void* O, float* lse,
                            void* workspace, hipStream_t s) {
    AttnParams prm;
    prm.Q = Q; prm.Kpre = Kpre; prm.Vpre = Vpre; prm.Kpriv = Kpriv; prm.Vpriv = Vpriv;
    prm.priv_len = priv_len;
    prm.O = O; prm.lse = lse;
    prm.B = d.B; prm.k = d.k; prm.R = d.k + 1; prm.Hq = d.Hq; prm.Hkv = d.Hkv; prm.G = d.Hq / d.Hkv;
    prm.GR = prm.G * prm.R; prm.D = d.D; prm.P = d.P; prm.Lmax = d.Lmax;
    prm.g_magic = (unsigned)((0x100000000ULL + (unsigned)prm.G - 1) / (unsigned)prm.G);  // G = 1 wraps to 0: handled where it is used
    const double scale = d.scale > 0.0f ? (double)d.scale : 1.0 / sqrt((double)d.D);
    prm.scale_log2 = (float)(scale * 1.4426950408889634074);
    prm.q_stride_b = d.q_stride_b; prm.q_stride_r = d.q_stride_r; prm.q_stride_h = d.q_stride_h;
    prm.kpre_stride_h = d.kpre_stride_h; prm.kpre_stride_t = d.kpre_stride_t;
    prm.kpriv_stride_b = d.kpriv_stride_b; prm.kpriv_stride_h = d.kpriv_stride_h; prm.kpriv_stride_t = d.kpriv_stride_t;
    prm.o_stride_b = d.o_stride_b; prm.o_stride_r = d.o_stride_r; prm.o_stride_h = d.o_stride_h;
    prm.tag = 0;
    const long long rows = (long long)d.B * prm.R * d.Hq;

    if (d.dtype == LOTTS_F32) {
        prm.plan = AttnPlan{};
        prm.ws = nullptr; prm.ws_bytes = 0; prm.off_o = prm.off_ml = 0; prm.counters = nullptr;
        if (d.D == 64)
            LOTTS_LAUNCH(attn_f32_kernel<64>, dim3((unsigned)rows), dim3(kAttnThreads), s, prm);
        else
            LOTTS_LAUNCH(attn_f32_kernel<128>, dim3((unsigned)rows), dim3(kAttnThreads), s, prm);
        return check_launch();
    }

    prm.plan = plan_attention(d);
    const AttnPlan& pl = prm.plan;
    size_t off_o, off_ml;
    const size_t total = workspace_layout(d, pl, &off_o, &off_ml);
    prm.ws = workspace;
    prm.ws_bytes = (unsigned)total;
    prm.off_o = (unsigned)off_o;
    prm.off_ml = (unsigned)off_ml;
    prm.counters = static_cast<unsigned long long*>(workspace);
    prm.tag = (g_call_tag.fetch_add(1, std::memory_order_relaxed) + 1) << kTagShift;
    const long long items = (long long)pl.n_pre_items + pl.n_priv_items;
    if (items > 0x7fffffffLL) return LOTTS_ERR_SHAPE;
    const dim3 grid((unsigned)items), block(kAttnThreads);
    const dim3 block2(2 * kAttnThreads);
    if (d.D == 128 && pl.nqt == 1) LOTTS_LAUNCH((attn_kernel<128, 1, 1>), grid, block, s, prm);
    else if (d.D == 128) LOTTS_LAUNCH((attn_kernel<128, 2, 2>), grid, block2, s, prm);
    else if (pl.nqt == 1) LOTTS_LAUNCH((attn_kernel<64, 1, 1>), grid, block, s, prm);
    else LOTTS_LAUNCH((attn_kernel<64, 2, 2>), grid, block2, s, prm);
    if (!pl.fused) {
        const int rc = check_launch();
        if (rc != LOTTS_OK) return rc;
        const dim3 mgrid((unsigned)((prm.GR * (d.D / 4) + kAttnThreads - 1) / kAttnThreads), (unsigned)(d.Hkv * d.B));
        if (d.D == 128) LOTTS_LAUNCH(attn_merge_kernel<128>, mgrid, block, s, prm);
        else LOTTS_LAUNCH(attn_merge_kernel<64>, mgrid, block, s, prm);
    }
    return check_launch();
}

// Pointer checks of both entry points (everything but the workspace).
static int check_pointers(const lotts_attn_desc& d, const void* Q, const void* Kpre, const void* Vpre, const void* Kpriv,
                          const void* Vpriv, const int32_t* priv_len, const void* O) {
    if (!Q || !Kpriv || !Vpriv || !priv_len || !O) return LOTTS_ERR_NULL;
    if (d.P > 0 && (!Kpre || !Vpre)) return LOTTS_ERR_NULL;
    const uintptr_t align_or = (uintptr_t)Q | (uintptr_t)Kpre | (uintptr_t)Vpre | (uintptr_t)Kpriv | (uintptr_t)Vpriv |
                               (uintptr_t)O;
    if (d.dtype == LOTTS_BF16 && (align_or & 15) != 0) return LOTTS_ERR_SHAPE;
    if ((align_or & 3) != 0) return LOTTS_ERR_SHAPE;
    return LOTTS_OK;
}

// ---------------------------------------------------------------------------------------------
// Scratch of the entry point that allocates nothing: arrival cells and partials live in a
// file-scope device array instead of a caller's workspace.  Each GPU holds its own copy of the array
// at its own address for the life of the process; in host code the array's name is only a handle, so
// the address is looked up once per device (with that device current) and the kernels get the
// looked-up pointer, exactly as they get a workspace pointer.  Zero-initialised when the code object
// is loaded, which is what the arrival cells want at first use.
// ---------------------------------------------------------------------------------------------
constexpr size_t kScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

static int scratch_of_current_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LOTTS_ERR_LAUNCH;
    void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {  // first call on this device; two threads racing here look up the same address
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return LOTTS_ERR_LAUNCH;
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return LOTTS_OK;
}

}  // namespace lotts

extern "C" size_t verify_attention_workspace_bytes(const lotts_attn_desc* desc) {
    using namespace lotts;
    lotts_attn_desc d;
    if (fill_desc(desc, &d) != LOTTS_OK) return 0;
    return workspace_need(d);
}

extern "C" int verify_attention(const lotts_attn_desc* desc, const void* Q, const void* Kpre, const void* Vpre,
                                const void* Kpriv, const void* Vpriv, const int32_t* priv_len, void* O, float* lse,
                                void* workspace, size_t workspace_bytes, void* stream) {
    using namespace lotts;
    lotts_attn_desc d;
    int rc = fill_desc(desc, &d);
    if (rc != LOTTS_OK) return rc;
    rc = check_pointers(d, Q, Kpre, Vpre, Kpriv, Vpriv, priv_len, O);
    if (rc != LOTTS_OK) return rc;
    if (!workspace) return LOTTS_ERR_NULL;
    const size_t need = workspace_need(d);
    if (need == 0) return LOTTS_ERR_SHAPE;  // a geometry whose partials the 32-bit offsets cannot address
    if (workspace_bytes < need) return LOTTS_ERR_WORKSPACE;
    if (((uintptr_t)workspace & (d.dtype == LOTTS_BF16 ? 15 : 3)) != 0) return LOTTS_ERR_SHAPE;
    return launch_attention(d, Q, Kpre, Vpre, Kpriv, Vpriv, priv_len, O, lse, workspace, (hipStream_t)stream);
}

extern "C" int verify_attention_noalloc(const lotts_attn_desc* desc, const void* Q, const void* Kpre, const void* Vpre,
                                        const void* Kpriv, const void* Vpriv, const int32_t* priv_len, void* O,
                                        float* lse, void* stream) {
    using namespace lotts;
    lotts_attn_desc d;
    int rc = fill_desc(desc, &d);
    if (rc != LOTTS_OK) return rc;
    rc = check_pointers(d, Q, Kpre, Vpre, Kpriv, Vpriv, priv_len, O);
    if (rc != LOTTS_OK) return rc;
    const size_t need = workspace_need(d);
    if (need == 0) return LOTTS_ERR_SHAPE;
    if (need > kScratchBytes) return LOTTS_ERR_WORKSPACE;  // beyond the built-in scratch: use verify_attention
    void* ptr = nullptr;
    rc = scratch_of_current_device(&ptr);
    if (rc != LOTTS_OK) return rc;
    return launch_attention(d, Q, Kpre, Vpre, Kpriv, Vpriv, priv_len, O, lse, ptr, (hipStream_t)stream);
}
