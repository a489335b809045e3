// kv_append: the K and V rows of the k + 1 new tokens of every branch go to the tail of the branch's private cache
// (paper Section 2: the drafted tokens are verified in one parallel forward of the target, so their keys and values
// join the cache before that forward's attention).  A strided copy in 16-byte pieces; one thread moves one piece of K
// and the same piece of V.
#include "lotts_common.h"

namespace lotts {

typedef unsigned a_u32x4 __attribute__((ext_vector_type(4)));

struct AppendParams {
    const unsigned char *Knew, *Vnew;
    unsigned char *Kpriv, *Vpriv;
    const int32_t* priv_len;
    long long new_b, new_r, new_h, priv_b, priv_h, priv_t;  // strides in bytes
    int B, R, Hkv, pieces, Lmax;                            // pieces: 16-byte pieces of a row of D elements
};

__global__ __launch_bounds__(256) void kv_append_kernel(const AppendParams p) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    const long long total = (long long)p.B * p.R * p.Hkv * p.pieces;
    if (i >= total) return;
    const int c = (int)(i % p.pieces);
    long long j = i / p.pieces;
    const int h = (int)(j % p.Hkv);
    j /= p.Hkv;
    const int r = (int)(j % p.R), b = (int)(j / p.R);
    // the source does not depend on the length: its loads go out together with the length's, one latency for all
    const long long src = b * p.new_b + r * p.new_r + h * p.new_h + c * 16LL;
    const a_u32x4 kv = *reinterpret_cast<const a_u32x4*>(p.Knew + src);
    const a_u32x4 vv = *reinterpret_cast<const a_u32x4*>(p.Vnew + src);
    const int t = p.priv_len[b] - p.R + r;  // position of new token r in the branch's private cache
    if (t < 0 || t >= p.Lmax) return;
    const long long dst = b * p.priv_b + h * p.priv_h + t * p.priv_t + c * 16LL;
    *reinterpret_cast<a_u32x4*>(p.Kpriv + dst) = kv;
    *reinterpret_cast<a_u32x4*>(p.Vpriv + dst) = vv;
}

}  // namespace lotts

extern "C" int kv_append(int32_t B, int32_t k, int32_t Hkv, int32_t D, lotts_dtype dtype, const void* Knew,
                         const void* Vnew, int64_t new_stride_b, int64_t new_stride_r, int64_t new_stride_h, void* Kpriv,
                         void* Vpriv, int64_t priv_stride_b, int64_t priv_stride_h, int64_t priv_stride_t, int32_t Lmax,
                         const int32_t* priv_len, void* stream) {
    using namespace lotts;
    if (dtype != LOTTS_BF16 && dtype != LOTTS_F32) return LOTTS_ERR_DTYPE;
    const long long es = dtype == LOTTS_BF16 ? 2 : 4;
    if (B < 1 || k < 0 || k > 255 || Hkv < 1 || D < 1 || Lmax < k + 1 || ((long long)D * es) % 16 != 0)
        return LOTTS_ERR_SHAPE;
    if (!Knew || !Vnew || !Kpriv || !Vpriv || !priv_len) return LOTTS_ERR_NULL;
    const int64_t strides[6] = {new_stride_b, new_stride_r, new_stride_h, priv_stride_b, priv_stride_h, priv_stride_t};
    for (int64_t s : strides)
        if (s < 0 || (s * es) % 16 != 0) return LOTTS_ERR_SHAPE;
    if (new_stride_h < D || priv_stride_t < D) return LOTTS_ERR_SHAPE;
    if ((((uintptr_t)Knew | (uintptr_t)Vnew | (uintptr_t)Kpriv | (uintptr_t)Vpriv) & 15) != 0) return LOTTS_ERR_SHAPE;
    AppendParams p;
    p.Knew = static_cast<const unsigned char*>(Knew);
    p.Vnew = static_cast<const unsigned char*>(Vnew);
    p.Kpriv = static_cast<unsigned char*>(Kpriv);
    p.Vpriv = static_cast<unsigned char*>(Vpriv);
    p.priv_len = priv_len;
    p.new_b = new_stride_b * es; p.new_r = new_stride_r * es; p.new_h = new_stride_h * es;
    p.priv_b = priv_stride_b * es; p.priv_h = priv_stride_h * es; p.priv_t = priv_stride_t * es;
    p.B = B; p.R = k + 1; p.Hkv = Hkv; p.pieces = (int)((long long)D * es / 16); p.Lmax = Lmax;
    const long long total = (long long)B * p.R * Hkv * p.pieces;
    if (total > (1LL << 40)) return LOTTS_ERR_SHAPE;
    LOTTS_LAUNCH(kv_append_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), (hipStream_t)stream, p);
    return check_launch();
}
