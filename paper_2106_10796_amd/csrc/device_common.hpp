// What every kernel shares: the chunk geometry, 128-bit loads and stores with ragged ends,
// widening of 16-bit gradients, and the error-feedback quantiser (Sec. 2.3, Sec. 3.4.1).
#pragma once

namespace {

constexpr unsigned kBlock = CDSGD_BLOCK;          // lanes per workgroup
constexpr unsigned kQpl = CDSGD_QPL;              // quads per lane
constexpr unsigned kChunkQuads = kBlock * kQpl;   // quads (= packed bytes) per chunk
constexpr unsigned kChunkElems = kChunkQuads * 4; // elements per chunk
static_assert(kQpl == 1 || kQpl == 2 || kQpl == 4, "a lane's packed bytes must fit one register");
static_assert(CDSGD_GRAD_F32 == 0 && CDSGD_GRAD_BF16 == 1 && CDSGD_GRAD_F16 == 2, "header and kernels agree");

typedef float f4 __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// 128-bit loads / stores, with the ragged end of a tensor handled per element
// ---------------------------------------------------------------------------
__device__ __forceinline__ f4 ld4(const float *base, unsigned qi)
{
    const f4 *p = reinterpret_cast<const f4 *>(base) + qi;
#if CDSGD_NT_LOAD
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}

__device__ __forceinline__ void st4(float *base, unsigned qi, f4 v)
{
    f4 *p = reinterpret_cast<f4 *>(base) + qi;
#if CDSGD_NT_STORE
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

// cnt = number of elements of this quad that exist (4 in the interior).
template <bool G>
__device__ __forceinline__ f4 ld4g(const float *base, unsigned qi, int cnt)
{
    if (!G || cnt == 4) return ld4(base, qi);
    f4 v = {0.0f, 0.0f, 0.0f, 0.0f};
    const float *p = base + 4u * qi;
    if (cnt > 0) v.x = p[0];
    if (cnt > 1) v.y = p[1];
    if (cnt > 2) v.z = p[2];
    return v;
}

template <bool G>
__device__ __forceinline__ void st4g(float *base, unsigned qi, int cnt, f4 v)
{
    if (!G || cnt == 4) {
        st4(base, qi, v);
        return;
    }
    float *p = base + 4u * qi;
    if (cnt > 0) p[0] = v.x;
    if (cnt > 1) p[1] = v.y;
    if (cnt > 2) p[2] = v.z;
}

// Gradient element types: fp32, or bf16 / fp16 widened exactly to fp32 on load
// (everything downstream of the load is the fp32 path).
constexpr int kGradF32 = 0, kGradBF16 = 1, kGradF16 = 2;

template <int GT>
__device__ __forceinline__ constexpr unsigned grad_bytes()
{
    return GT == kGradF32 ? 4u : 2u;
}

typedef unsigned u2 __attribute__((ext_vector_type(2)));

template <int GT>
__device__ __forceinline__ float widen16(unsigned h)  // h: the 16-bit pattern in the low half
{
    if (GT == kGradBF16) return __builtin_bit_cast(float, h << 16);
    return (float)__builtin_bit_cast(_Float16, (unsigned short)h);
}

// One quad of a gradient buffer; `base` is the chunk's first element.
template <bool G, int GT>
__device__ __forceinline__ f4 ldgrad(const void *base, unsigned qi, int cnt)
{
    if (GT == kGradF32) return ld4g<G>(static_cast<const float *>(base), qi, cnt);
    if (!G || cnt == 4) {
        const u2 *p = static_cast<const u2 *>(base) + qi;
#if CDSGD_NT_LOAD
        const u2 v = __builtin_nontemporal_load(p);
#else
        const u2 v = *p;
#endif
        return f4{widen16<GT>(v.x & 0xFFFFu), widen16<GT>(v.x >> 16), widen16<GT>(v.y & 0xFFFFu),
                  widen16<GT>(v.y >> 16)};
    }
    f4 v = {0.0f, 0.0f, 0.0f, 0.0f};
    const unsigned short *p = static_cast<const unsigned short *>(base) + 4u * qi;
    if (cnt > 0) v.x = widen16<GT>(p[0]);
    if (cnt > 1) v.y = widen16<GT>(p[1]);
    if (cnt > 2) v.z = widen16<GT>(p[2]);
    return v;
}

template <int GT>
__device__ __forceinline__ const void *grad_at(const void *grad, size_t quad0)
{
    return static_cast<const char *>(grad) + quad0 * (4u * grad_bytes<GT>());
}

template <bool G>
__device__ __forceinline__ int quad_count(unsigned rem_elems, unsigned qi)
{
    if (!G) return 4;
    int c = (int)rem_elems - (int)(4u * qi);
    return c < 0 ? 0 : (c > 4 ? 4 : c);
}

// ---------------------------------------------------------------------------
// a1 + a2: error-feedback threshold quantiser (Sec. 2.3, Sec. 3.4.1)
// ---------------------------------------------------------------------------
// a = r + g; |a| >= t sends sign(a)*t and keeps the rest.  `sent` is what the
// code stands for (+t, -t or +0); a - sent is bit-identical to a - t, a + t and
// a in the three cases.  Returns the 2-bit code (1 = +t, 2 = -t).
__device__ __forceinline__ unsigned quantize1(float g, float &r, float t, float &sent)
{
    const float a = r + g;
    const bool pos = a >= t;
    const bool neg = a <= -t;
    sent = pos ? t : (neg ? -t : 0.0f);
    r = a - sent;
    return pos ? 1u : (neg ? 2u : 0u);
}

// One quad: residual updated in place, returns the packed byte.
__device__ __forceinline__ unsigned quantize_quad(const f4 g, f4 &r, float t, f4 &sent)
{
    float s0, s1, s2, s3, r0 = r.x, r1 = r.y, r2 = r.z, r3 = r.w;
    const unsigned c0 = quantize1(g.x, r0, t, s0);
    const unsigned c1 = quantize1(g.y, r1, t, s1);
    const unsigned c2 = quantize1(g.z, r2, t, s2);
    const unsigned c3 = quantize1(g.w, r3, t, s3);
    r = f4{r0, r1, r2, r3};
    sent = f4{s0, s1, s2, s3};
    return c0 | (c1 << 2) | (c2 << 4) | (c3 << 6);
}

}  // namespace
