// gfx950 kernels of the HALoS server-side update path.
//
// Every step of the path is an elementwise read-modify-write over parameter-sized arrays, so the
// kernels are bandwidth machines: each wavefront issues 128-bit accesses that cover 1 KiB of
// consecutive addresses per stream, a workgroup keeps UNROLL of them in flight per stream before it
// consumes any, and a persistent grid walks a tile table so that one launch covers the whole tensor
// list.  There is no contraction anywhere, hence no MFMA and no LDS staging.
//
// Arithmetic is written with explicit single-rounding intrinsics in one fixed order, so results do
// not depend on compiler contraction settings:
//     m1 = fma(beta, m, g);  u = fma(beta, m1, cg * g);  s = eta * u;  x = x - s;  acc = acc + s
//     merge: theta = fma(alpha, Theta_i, keep * theta)
//     delayed momentum: b1 = b + g;  gp = (cg/d) * g;  s = eta * gp,  or at a refresh
//                       m1 = fma(beta, m, b1 * (1/d));  s = eta * fma(beta, m1, gp)
#include <hip/hip_runtime.h>

#include <atomic>

#include "kernels.hpp"

namespace halos {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));

// Pointers read from a table in memory are generic ("flat") to the compiler.  Everything this
// library touches is global device memory, so say so: global_load/global_store instead of flat_*.
#define HALOS_GLOBAL __attribute__((address_space(1)))
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef HALOS_GLOBAL float gf32;
typedef HALOS_GLOBAL unsigned short gu16;       // bfloat16 bit patterns
typedef HALOS_GLOBAL _Float16 gf16;             // IEEE half
typedef HALOS_GLOBAL f32x4 gf32x4;
typedef HALOS_GLOBAL u16x4 gu16x4;
typedef HALOS_GLOBAL f16x4 gf16x4;

__device__ __forceinline__ gf32 *to_global(float *p) { return (gf32 *)p; }
__device__ __forceinline__ const gf32 *to_global(const float *p) { return (const gf32 *)p; }
__device__ __forceinline__ const gu16 *to_global(const unsigned short *p) { return (const gu16 *)p; }
__device__ __forceinline__ const gf16 *to_global(const _Float16 *p) { return (const gf16 *)p; }

template <bool NT>
__device__ __forceinline__ f32x4 ld4(const gf32 *p) {
    const gf32x4 *q = (const gf32x4 *)p;
    if constexpr (NT) return __builtin_nontemporal_load(q);
    else return *q;
}

template <bool NT>
__device__ __forceinline__ void st4(gf32 *p, f32x4 v) {
    gf32x4 *q = (gf32x4 *)p;
    if constexpr (NT) __builtin_nontemporal_store(v, q);
    else *q = v;
}

__device__ __forceinline__ float bf16_up(unsigned short bits) {     // bfloat16 = upper half of a binary32
    return __uint_as_float(static_cast<uint32_t>(bits) << 16);
}

// Four consecutive delta elements as fp32, from an fp32 or a bf16 tensor.
template <bool NT>
__device__ __forceinline__ f32x4 ldg4(const gf32 *p) { return ld4<NT>(p); }

template <bool NT>
__device__ __forceinline__ f32x4 ldg4(const gu16 *p) {
    const gu16x4 *q = (const gu16x4 *)p;
    u16x4 b;
    if constexpr (NT) b = __builtin_nontemporal_load(q);
    else b = *q;
    f32x4 r;
    r[0] = bf16_up(b[0]); r[1] = bf16_up(b[1]); r[2] = bf16_up(b[2]); r[3] = bf16_up(b[3]);
    return r;
}

template <bool NT>
__device__ __forceinline__ f32x4 ldg4(const gf16 *p) {          // half -> float is exact for every half value
    const gf16x4 *q = (const gf16x4 *)p;
    f16x4 h;
    if constexpr (NT) h = __builtin_nontemporal_load(q);
    else h = *q;
    f32x4 r;
    r[0] = static_cast<float>(h[0]); r[1] = static_cast<float>(h[1]); r[2] = static_cast<float>(h[2]); r[3] = static_cast<float>(h[3]);
    return r;
}

__device__ __forceinline__ float ldg1(const gf32 *p) { return *p; }
__device__ __forceinline__ float ldg1(const gu16 *p) { return bf16_up(*p); }
__device__ __forceinline__ float ldg1(const gf16 *p) { return static_cast<float>(*p); }

// Momentum kept in bfloat16 (MB): the array holds 16-bit patterns; a new momentum is rounded to bfloat16 (nearest,
// ties to even, decided on the binary32 value; a NaN becomes the quiet NaN 0x7FC0) BEFORE it enters the step, so the
// value that is used is the value that is stored.  bf16_round returns that value as a float (low half zero).
__device__ __forceinline__ float bf16_round(float v) {
    const uint32_t u = __float_as_uint(v);
    const uint32_t r = (u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u;
    return __uint_as_float((u & 0x7FFFFFFFu) > 0x7F800000u ? 0x7FC00000u : r);
}

template <bool MB> struct MomentumElem { typedef gf32 type; };
template <> struct MomentumElem<true> { typedef gu16 type; };
template <bool MB>
__device__ __forceinline__ typename MomentumElem<MB>::type *momentum_ptr(float *p) {
    return (typename MomentumElem<MB>::type *)p;
}

template <bool NT>
__device__ __forceinline__ void stm4(gf32 *p, f32x4 v) { st4<NT>(p, v); }
template <bool NT>
__device__ __forceinline__ void stm4(gu16 *p, f32x4 v) {          // v holds bfloat16 values: keep the upper halves
    u16x4 b;
    b[0] = static_cast<unsigned short>(__float_as_uint(v[0]) >> 16); b[1] = static_cast<unsigned short>(__float_as_uint(v[1]) >> 16);
    b[2] = static_cast<unsigned short>(__float_as_uint(v[2]) >> 16); b[3] = static_cast<unsigned short>(__float_as_uint(v[3]) >> 16);
    gu16x4 *q = (gu16x4 *)p;
    if constexpr (NT) __builtin_nontemporal_store(b, q);
    else *q = b;
}
__device__ __forceinline__ void stm1(gf32 *p, float v) { *p = v; }
__device__ __forceinline__ void stm1(gu16 *p, float v) { *p = static_cast<unsigned short>(__float_as_uint(v) >> 16); }

// The same four delta elements as they lie in memory, and their upcast as a separate step: a pass that loads several
// deltas under (uniform) branches issues all its loads first and converts afterwards, instead of waiting per delta.
template <bool NT> __device__ __forceinline__ f32x4 ldraw4(const gf32 *p) { return ld4<NT>(p); }
template <bool NT> __device__ __forceinline__ u16x4 ldraw4(const gu16 *p) {
    const gu16x4 *q = (const gu16x4 *)p;
    if constexpr (NT) return __builtin_nontemporal_load(q);
    else return *q;
}
template <bool NT> __device__ __forceinline__ f16x4 ldraw4(const gf16 *p) {
    const gf16x4 *q = (const gf16x4 *)p;
    if constexpr (NT) return __builtin_nontemporal_load(q);
    else return *q;
}
__device__ __forceinline__ f32x4 up4(f32x4 v) { return v; }
__device__ __forceinline__ f32x4 up4(u16x4 b) {
    f32x4 r;
    r[0] = bf16_up(b[0]); r[1] = bf16_up(b[1]); r[2] = bf16_up(b[2]); r[3] = bf16_up(b[3]);
    return r;
}
__device__ __forceinline__ f32x4 up4(f16x4 h) {
    f32x4 r;
    r[0] = static_cast<float>(h[0]); r[1] = static_cast<float>(h[1]); r[2] = static_cast<float>(h[2]); r[3] = static_cast<float>(h[3]);
    return r;
}

__device__ __forceinline__ f32x4 sub4(f32x4 a, f32x4 b);

// The pseudo-gradient of four consecutive elements: read from the worker's delta tensor, or (FROM_END) formed here
// as start - end from the worker's start model (the buffer the server filled at the worker's last pull) and the end
// model the worker sent (the delta of Alg. 1's worker block, formed on the server, sign flipped).
// ... times the caller's scalar on this delta (gw = 1 is exact and changes nothing).
__device__ __forceinline__ f32x4 scale4(float w, f32x4 v);

template <bool FROM_END, bool NT, typename GP>
__device__ __forceinline__ f32x4 grad4(const GP *g, const gf32 *start, uint32_t off, float gw) {
    if constexpr (FROM_END) return scale4(gw, sub4(ld4<NT>(start + off), ld4<NT>(g + off)));
    else return scale4(gw, ldg4<NT>(g + off));
}

template <bool FROM_END, typename GP>
__device__ __forceinline__ float grad1(const GP *g, const gf32 *start, uint32_t k, float gw) {
    if constexpr (FROM_END) return __fmul_rn(gw, __fsub_rn(start[k], ldg1(g + k)));
    else return __fmul_rn(gw, ldg1(g + k));
}

// ModelUpdate (App. E) on one element; returns the step that was subtracted from x.
template <bool MB = false>
__device__ __forceinline__ float model_update(float &x, float &m, float g, float eta, float beta, float cg) {
    m = __fmaf_rn(beta, m, g);
    if constexpr (MB) m = bf16_round(m);
    const float u = __fmaf_rn(beta, m, __fmul_rn(cg, g));
    const float s = __fmul_rn(eta, u);
    x = __fsub_rn(x, s);
    return s;
}


// The same on four lanes of a 128-bit access (vector elements cannot be bound to references).
template <bool MB = false>
__device__ __forceinline__ f32x4 model_update4(f32x4 &x, f32x4 &m, f32x4 g, float eta, float beta, float cg) {
    f32x4 s;
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        float xi = x[i], mi = m[i];
        s[i] = model_update<MB>(xi, mi, g[i], eta, beta, cg);
        x[i] = xi;
        m[i] = mi;
    }
    return s;
}

__device__ __forceinline__ f32x4 add4(f32x4 a, f32x4 b) {
    f32x4 r;
#pragma unroll
    for (int i = 0; i < VEC; ++i) r[i] = __fadd_rn(a[i], b[i]);
    return r;
}

// The merge of Alg. 1's LPS block in the two-product form: exact for alpha = 0 (keep = 1) and alpha = 1 (keep = 0).
__device__ __forceinline__ float merge1(float theta, float global, float alpha, float keep) {
    return __fmaf_rn(alpha, global, __fmul_rn(keep, theta));
}

__device__ __forceinline__ f32x4 merge4(f32x4 theta, f32x4 global, float alpha, float keep) {
    f32x4 r;
#pragma unroll
    for (int i = 0; i < VEC; ++i) r[i] = merge1(theta[i], global[i], alpha, keep);
    return r;
}

// Sum of squares of four lanes, in fp32 (16 values per thread and tile are added in fp32, tiles in fp64).
__device__ __forceinline__ float sumsq4(f32x4 v, float q) {
#pragma unroll
    for (int i = 0; i < VEC; ++i) q = __fmaf_rn(v[i], v[i], q);
    return q;
}

__device__ __forceinline__ f32x4 sub4(f32x4 a, f32x4 b) {
    f32x4 r;
#pragma unroll
    for (int i = 0; i < VEC; ++i) r[i] = __fsub_rn(a[i], b[i]);
    return r;
}

__device__ __forceinline__ f32x4 scale4(float w, f32x4 v) {
    f32x4 r;
#pragma unroll
    for (int i = 0; i < VEC; ++i) r[i] = __fmul_rn(w, v[i]);
    return r;
}

// Wavefront reduction (64 lanes, shuffles), then the four wavefronts of the workgroup through LDS.
// Every thread of the workgroup must call it.  Thread 0 stores the workgroup's total.
__device__ __forceinline__ void block_sum_store(double v, double *dst) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    __shared__ double wave_total[BLOCK_THREADS / 64];
    if ((threadIdx.x & 63) == 0) wave_total[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
#pragma unroll
        for (int w = 0; w < BLOCK_THREADS / 64; ++w) t += wave_total[w];
        *dst = t;
    }
}

// ---------------------------------------------------------------------------------------------
// S1: worker-delta step of a local server.
// THIRD says what happens to the server's third buffer: 0 untouched, 1 running accumulation (acc <- acc + s),
// 2 it holds the snapshot theta_{t_last} and this update completes the accumulation: it is overwritten with
// G = theta_{t_last} - theta_t (Alg. 1's Delta, sign flipped), 3 the accumulation restarts here: acc <- 0 + s without
// reading what the buffer held (the merge before it did not clear it).
// gw is the caller's scalar on this delta: the update is applied to gw * g.
// With PULL the updated model is also written to a second tensor list (the buffer the worker starts
// its next round from: ModelUpdate and "schedule the worker" of Alg. 1 in one pass instead of an update pass plus a copy pass).
// With NORM every workgroup also leaves the sum of g^2 over its tiles in partials[blockIdx.x].
// With FROM_END (needs PULL) the delta tensors hold the worker's end model and pull_tab its start model.
// With MB the momentum tensors hold bfloat16 (see bf16_round).
template <typename GT, int THIRD, bool NT, bool PULL, bool NORM, bool FROM_END = false, bool MB = false>
__global__ void __launch_bounds__(BLOCK_THREADS)
lps_update_kernel(const Tile *__restrict__ tiles, uint32_t tile_lo, uint32_t tile_hi, uint32_t tensor_base,
                  float *const *__restrict__ theta_tab, float *const *__restrict__ m_tab,
                  float *const *__restrict__ acc_tab, float *const *__restrict__ pull_tab, PtrArgs gargs,
                  float eta, float beta, float cg, float gw, double *__restrict__ partials) {
    static_assert(!FROM_END || (PULL && sizeof(GT) == 4), "an end model is fp32 and needs the worker's start model");
    constexpr bool LOAD_THIRD = THIRD == 1 || THIRD == 2;
    const uint32_t tid = threadIdx.x;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    double norm_acc = 0.0;
    for (uint32_t t = tile_lo + blockIdx.x; t < tile_hi; t += gridDim.x) {
        const Tile tl = tiles[t];
        const uint32_t tensor = tl.tensor;
        gf32 *th = to_global(theta_tab[tensor]) + tl.start;
        auto *mm = momentum_ptr<MB>(m_tab[tensor]) + tl.start;
        gf32 *ac = THIRD != 0 ? to_global(acc_tab[tensor]) + tl.start : nullptr;
        gf32 *pd = PULL ? to_global(pull_tab[tensor]) + tl.start : nullptr;
        const auto *g = to_global(static_cast<const GT *>(gargs.p[tensor - tensor_base])) + tl.start;
        if (tl.len == TILE_ELEMS) {
            f32x4 gv[UNROLL], mv[UNROLL], tv[UNROLL], av[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t off = (u * BLOCK_THREADS + tid) * VEC;
                gv[u] = grad4<FROM_END, NT>(g, pd, off, gw);
                mv[u] = ldg4<NT>(mm + off);
                tv[u] = ld4<NT>(th + off);
                if constexpr (LOAD_THIRD) av[u] = ld4<NT>(ac + off);
            }
            if constexpr (NORM) {
                float q = 0.f;
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) q = sumsq4(gv[u], q);
                norm_acc += static_cast<double>(q);
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t off = (u * BLOCK_THREADS + tid) * VEC;
                const f32x4 s = model_update4<MB>(tv[u], mv[u], gv[u], eta, beta, cg);
                stm4<NT>(mm + off, mv[u]);
                st4<NT>(th + off, tv[u]);
                if constexpr (PULL) st4<NT>(pd + off, tv[u]);
                if constexpr (THIRD == 1) st4<NT>(ac + off, add4(av[u], s));
                if constexpr (THIRD == 2) st4<NT>(ac + off, sub4(av[u], tv[u]));
                if constexpr (THIRD == 3) st4<NT>(ac + off, add4(zero, s));
            }
        } else {
            const uint32_t len = tl.len;
            for (uint32_t off = tid * VEC; off < len; off += BLOCK_THREADS * VEC) {
                if (off + VEC <= len) {
                    f32x4 gv = grad4<FROM_END, NT>(g, pd, off, gw), mv = ldg4<NT>(mm + off), tv = ld4<NT>(th + off);
                    if constexpr (NORM) norm_acc += static_cast<double>(sumsq4(gv, 0.f));
                    const f32x4 s = model_update4<MB>(tv, mv, gv, eta, beta, cg);
                    stm4<NT>(mm + off, mv);
                    st4<NT>(th + off, tv);
                    if constexpr (PULL) st4<NT>(pd + off, tv);
                    if constexpr (THIRD == 1) st4<NT>(ac + off, add4(ld4<NT>(ac + off), s));
                    if constexpr (THIRD == 2) st4<NT>(ac + off, sub4(ld4<NT>(ac + off), tv));
                    if constexpr (THIRD == 3) st4<NT>(ac + off, add4(zero, s));
                } else {
                    for (uint32_t k = off; k < len; ++k) {      // ragged tail: fewer than 4 elements
                        float mv = ldg1(mm + k), tv = th[k];
                        const float gk = grad1<FROM_END>(g, pd, k, gw);
                        if constexpr (NORM) norm_acc += static_cast<double>(__fmul_rn(gk, gk));
                        const float s = model_update<MB>(tv, mv, gk, eta, beta, cg);
                        stm1(mm + k, mv); th[k] = tv;
                        if constexpr (PULL) pd[k] = tv;
                        if constexpr (THIRD == 1) ac[k] = __fadd_rn(ac[k], s);
                        if constexpr (THIRD == 2) ac[k] = __fsub_rn(ac[k], tv);
                        if constexpr (THIRD == 3) ac[k] = __fadd_rn(0.f, s);
                    }
                }
            }
        }
    }
    if constexpr (NORM) block_sum_store(norm_acc, partials + blockIdx.x);
}

// ---------------------------------------------------------------------------------------------
// S1 over several deltas in one pass (see kernels.hpp, launch_lps_update_multi).  SEQ: apply them one after the other;
// otherwise average them and apply the mean once.  THIRD as in lps_update_kernel; under SEQ the first n_acc deltas
// count towards the accumulated update, and with THIRD = 2 the n_acc-th turns the snapshot into theta_{t_last} - theta_t.
// With MB the momentum tensors hold bfloat16 and the momentum is rounded after every one of the updates, as in single steps.
// With MERGE (SEQ, THIRD 1 or 2) the third buffer arrives holding the returned global model: merge it into theta first,
// then restart the accumulation (THIRD 1: from zero; THIRD 2: the merged model is the new snapshot).
template <typename GT, bool SEQ, int THIRD, bool PULL, bool MB = false, bool MERGE = false>
__global__ void __launch_bounds__(BLOCK_THREADS)
lps_update_multi_kernel(const Tile *__restrict__ tiles, uint32_t tile_lo, uint32_t tile_hi,
                        float *const *__restrict__ theta_tab, float *const *__restrict__ m_tab,
                        float *const *__restrict__ acc_tab, MultiArgs a, float eta, float beta, float cg, float inv_n) {
    static_assert(!MERGE || (SEQ && (THIRD == 1 || THIRD == 2)), "a merge-first pass is sequential and rewrites the third buffer");
    constexpr bool NT = true;
    constexpr bool LOAD_THIRD = THIRD == 1 || THIRD == 2;
    const uint32_t tid = threadIdx.x;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    const int n_in = a.n_in, n_acc = a.n_acc;
    for (uint32_t t = tile_lo + blockIdx.x; t < tile_hi; t += gridDim.x) {
        const Tile tl = tiles[t];
        const uint32_t tensor = tl.tensor;
        gf32 *th = to_global(theta_tab[tensor]) + tl.start;
        auto *mm = momentum_ptr<MB>(m_tab[tensor]) + tl.start;
        gf32 *ac = THIRD != 0 ? to_global(acc_tab[tensor]) + tl.start : nullptr;
        decltype(to_global(static_cast<const GT *>(nullptr))) g[MAX_MULTI];
        gf32 *pd[MAX_MULTI];
#pragma unroll
        for (int i = 0; i < MAX_MULTI; ++i) {
            g[i] = i < n_in ? to_global(reinterpret_cast<const GT *>(a.delta[i][tensor])) + tl.start : nullptr;
            pd[i] = (PULL && i < n_in && a.pull[i]) ? to_global(a.pull[i][tensor]) + tl.start : nullptr;
        }
        if (tl.len == TILE_ELEMS) {
            decltype(ldraw4<NT>(g[0])) gv[MAX_MULTI][UNROLL];      // as loaded; upcast and weighted where they are used
            f32x4 mv[UNROLL], tv[UNROLL], av[UNROLL];
#pragma unroll
            for (int i = 0; i < MAX_MULTI; ++i)
                if (i < n_in) {
#pragma unroll
                    for (int u = 0; u < UNROLL; ++u) gv[i][u] = ldraw4<NT>(g[i] + (u * BLOCK_THREADS + tid) * VEC);
                }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t off = (u * BLOCK_THREADS + tid) * VEC;
                mv[u] = ldg4<NT>(mm + off);
                tv[u] = ld4<NT>(th + off);
                av[u] = LOAD_THIRD ? ld4<NT>(ac + off) : zero;
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t off = (u * BLOCK_THREADS + tid) * VEC;
                if constexpr (MERGE) {
                    tv[u] = merge4(tv[u], av[u], a.alpha, a.keep);
                    av[u] = THIRD == 2 ? tv[u] : zero;
                }
                if constexpr (SEQ) {
#pragma unroll
                    for (int i = 0; i < MAX_MULTI; ++i)
                        if (i < n_in) {
                            const f32x4 s = model_update4<MB>(tv[u], mv[u], scale4(a.w[i], up4(gv[i][u])), eta, beta, cg);
                            if constexpr (THIRD == 1 || THIRD == 3) { if (i < n_acc) av[u] = add4(av[u], s); }
                            if constexpr (THIRD == 2) { if (i + 1 == n_acc) av[u] = sub4(av[u], tv[u]); }
                            if constexpr (PULL) { if (pd[i]) st4<NT>(pd[i] + off, tv[u]); }
                        }
                } else {
                    f32x4 sum = scale4(a.w[0], up4(gv[0][u]));
#pragma unroll
                    for (int i = 1; i < MAX_MULTI; ++i)
                        if (i < n_in) sum = add4(sum, scale4(a.w[i], up4(gv[i][u])));
                    const f32x4 s = model_update4<MB>(tv[u], mv[u], scale4(inv_n, sum), eta, beta, cg);
                    if constexpr (THIRD == 1 || THIRD == 3) av[u] = add4(av[u], s);
                    if constexpr (THIRD == 2) av[u] = sub4(av[u], tv[u]);
                }
                stm4<NT>(mm + off, mv[u]);
                st4<NT>(th + off, tv[u]);
                if constexpr (THIRD != 0) st4<NT>(ac + off, av[u]);
            }
        } else {                                    // a ragged tile: element by element
            const uint32_t len = tl.len;
            for (uint32_t k = tid; k < len; k += BLOCK_THREADS) {
                float mk = ldg1(mm + k), tk = th[k], ak = LOAD_THIRD ? ac[k] : 0.f;
                if constexpr (MERGE) {
                    tk = merge1(tk, ak, a.alpha, a.keep);
                    ak = THIRD == 2 ? tk : 0.f;
                }
                if constexpr (SEQ) {
                    for (int i = 0; i < n_in; ++i) {
                        const float s = model_update<MB>(tk, mk, __fmul_rn(a.w[i], ldg1(g[i] + k)), eta, beta, cg);
                        if constexpr (THIRD == 1 || THIRD == 3) { if (i < n_acc) ak = __fadd_rn(ak, s); }
                        if constexpr (THIRD == 2) { if (i + 1 == n_acc) ak = __fsub_rn(ak, tk); }
                        if constexpr (PULL) { if (pd[i]) pd[i][k] = tk; }
                    }
                } else {
                    float sum = __fmul_rn(a.w[0], ldg1(g[0] + k));
                    for (int i = 1; i < n_in; ++i) sum = __fadd_rn(sum, __fmul_rn(a.w[i], ldg1(g[i] + k)));
                    const float s = model_update<MB>(tk, mk, __fmul_rn(inv_n, sum), eta, beta, cg);
                    if constexpr (THIRD == 1 || THIRD == 3) ak = __fadd_rn(ak, s);
                    if constexpr (THIRD == 2) ak = __fsub_rn(ak, tk);
                }
                stm1(mm + k, mk); th[k] = tk;
                if constexpr (THIRD != 0) ac[k] = ak;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// S3: global-server step.  G and out may alias.  With MB the momentum tensors hold bfloat16 (see bf16_round).
template <bool NT, bool MB = false>
__global__ void __launch_bounds__(BLOCK_THREADS)
gps_update_kernel(const Tile *__restrict__ tiles, uint32_t tile_lo, uint32_t tile_hi,
                  float *const *__restrict__ Theta_tab, float *const *__restrict__ M_tab,
                  float *const *G_tab, float *const *out_tab, float eta, float beta, float cg) {
    const uint32_t tid = threadIdx.x;
    for (uint32_t t = tile_lo + blockIdx.x; t < tile_hi; t += gridDim.x) {
        const Tile tl = tiles[t];
        const uint32_t tensor = tl.tensor;
        gf32 *Th = to_global(Theta_tab[tensor]) + tl.start;
        auto *Mm = momentum_ptr<MB>(M_tab[tensor]) + tl.start;
        const gf32 *G = to_global(G_tab[tensor]) + tl.start;
        gf32 *out = to_global(out_tab[tensor]) + tl.start;
        if (tl.len == TILE_ELEMS) {
            f32x4 gv[UNROLL], mv[UNROLL], tv[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t off = (u * BLOCK_THREADS + tid) * VEC;
                gv[u] = ld4<NT>(G + off);
                mv[u] = ldg4<NT>(Mm + off);
                tv[u] = ld4<NT>(Th + off);
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t off = (u * BLOCK_THREADS + tid) * VEC;
                model_update4<MB>(tv[u], mv[u], gv[u], eta, beta, cg);
                stm4<NT>(Mm + off, mv[u]);
                st4<NT>(Th + off, tv[u]);
                st4<NT>(out + off, tv[u]);
            }
        } else {
            const uint32_t len = tl.len;
            for (uint32_t off = tid * VEC; off < len; off += BLOCK_THREADS * VEC) {
                if (off + VEC <= len) {
                    f32x4 gv = ld4<NT>(G + off), mv = ldg4<NT>(Mm + off), tv = ld4<NT>(Th + off);
                    model_update4<MB>(tv, mv, gv, eta, beta, cg);
                    stm4<NT>(Mm + off, mv);
                    st4<NT>(Th + off, tv);
                    st4<NT>(out + off, tv);
                } else {
                    for (uint32_t k = off; k < len; ++k) {
                        float mv = ldg1(Mm + k), tv = Th[k];
                        model_update<MB>(tv, mv, G[k], eta, beta, cg);
                        stm1(Mm + k, mv); Th[k] = tv; out[k] = tv;
                    }
                }
            }
        }
    }
}

// S3 without global momentum (beta_g = 0, the setting of Sec. 5.4 for non-i.i.d. data): the momentum array is neither
// read nor written, Theta <- Theta - eta (cg G).  Same bits as gps_update_kernel at beta = 0 (where m = G and the
// momentum term is an exact zero), up to the sign of an exact zero.  G and out may alias.
template <bool NT>
__global__ void __launch_bounds__(BLOCK_THREADS)
gps_update_nomom_kernel(const Tile *__restrict__ tiles, uint32_t tile_lo, uint32_t tile_hi,
                        float *const *__restrict__ Theta_tab, float *const *G_tab, float *const *out_tab, float eta, float cg) {
    const uint32_t tid = threadIdx.x;
    for (uint32_t t = tile_lo + blockIdx.x; t < tile_hi; t += gridDim.x) {
        const Tile tl = tiles[t];
        const uint32_t tensor = tl.tensor;
        gf32 *Th = to_global(Theta_tab[tensor]) + tl.start;
        const gf32 *G = to_global(G_tab[tensor]) + tl.start;
        gf32 *out = to_global(out_tab[tensor]) + tl.start;
        if (tl.len == TILE_ELEMS) {
            f32x4 gv[UNROLL], tv[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t off = (u * BLOCK_THREADS + tid) * VEC;
                gv[u] = ld4<NT>(G + off);
                tv[u] = ld4<NT>(Th + off);
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t off = (u * BLOCK_THREADS + tid) * VEC;
                const f32x4 nt = sub4(tv[u], scale4(eta, scale4(cg, gv[u])));
                st4<NT>(Th + off, nt);
                st4<NT>(out + off, nt);
            }
        } else {
            const uint32_t len = tl.len;
            for (uint32_t off = tid * VEC; off < len; off += BLOCK_THREADS * VEC) {
                if (off + VEC <= len) {
                    const f32x4 nt = sub4(ld4<NT>(Th + off), scale4(eta, scale4(cg, ld4<NT>(G + off))));
                    st4<NT>(Th + off, nt);
                    st4<NT>(out + off, nt);
                } else {
                    for (uint32_t k = off; k < len; ++k) {
                        const float nt = __fsub_rn(Th[k], __fmul_rn(eta, __fmul_rn(cg, G[k])));
                        Th[k] = nt; out[k] = nt;
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Delayed Nesterov momentum (Sec. 5.1; App. D, delays d_l and d_g).  A server handles its updates in cycles
// of d: every update adds g to a buffer and steps the model by eta (cg/d) g; the last one of a cycle also
// refreshes the momentum from the buffer's mean and applies it.  RULE says where in the cycle an update is:
//   CYCLE_FIRST    opens a cycle: buffer <- g (the buffer is not read)
//   CYCLE_INNER    buffer <- buffer + g
//   CYCLE_REFRESH  closes it: m <- beta m + (buffer + g)/d, applied; the buffer is not written
// Only a refresh touches the momentum.

template <int RULE>
__device__ __forceinline__ float delayed_update(float &x, float &m, float &b, float g, float eta, float beta, float cgd,
                                                float inv_d) {
    const float b1 = RULE == CYCLE_FIRST ? g : __fadd_rn(b, g);
    const float gp = __fmul_rn(cgd, g);
    float u = gp;
    if constexpr (RULE == CYCLE_REFRESH) {
        m = __fmaf_rn(beta, m, __fmul_rn(b1, inv_d));
        u = __fmaf_rn(beta, m, gp);
    }
    b = b1;
    const float s = __fmul_rn(eta, u);
    x = __fsub_rn(x, s);
    return s;
}

template <int RULE>
__device__ __forceinline__ f32x4 delayed_update4(f32x4 &x, f32x4 &m, f32x4 &b, f32x4 g, float eta, float beta, float cgd,
                                                 float inv_d) {
    f32x4 s;
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        float xi = x[i], mi = m[i], bi = b[i];
        s[i] = delayed_update<RULE>(xi, mi, bi, g[i], eta, beta, cgd, inv_d);
        x[i] = xi;
        m[i] = mi;
        b[i] = bi;
    }
    return s;
}

// S1 under the delayed rule.  THIRD and PULL as in lps_update_kernel; accesses are non-temporal.
// MERGE: the third buffer arrives holding the returned global model Theta_i; each element is merged first
// (theta <- alpha Theta_i + keep theta, the merge of Alg. 1's LPS block) and the accumulation restarts with this update:
// THIRD 1 the third buffer leaves as 0 + s; THIRD 2 (snapshot form, this update completes the accumulation) as
// merged - updated; THIRD 4 (snapshot form, it does not) as the merged model, the new snapshot.
template <typename GT, int THIRD, bool PULL, int RULE, bool FROM_END, bool NORM, bool MERGE = false>
__global__ void __launch_bounds__(BLOCK_THREADS)
lps_update_delayed_kernel(const Tile *__restrict__ tiles, uint32_t tile_lo, uint32_t tile_hi, uint32_t tensor_base,
                          float *const *__restrict__ theta_tab, float *const *__restrict__ m_tab,
                          float *const *__restrict__ buf_tab, float *const *__restrict__ acc_tab,
                          float *const *__restrict__ pull_tab, PtrArgs gargs, float eta, float beta, float cgd,
                          float inv_d, float gw, double *__restrict__ partials, float alpha, float keep) {
    static_assert(!FROM_END || (PULL && sizeof(GT) == 4), "an end model is fp32 and needs the worker's start model");
    static_assert(MERGE ? (THIRD == 1 || THIRD == 2 || THIRD == 4) : THIRD != 4, "THIRD 4 exists only for a merge-first pass");
    constexpr bool NT = true;
    constexpr bool LOAD_THIRD = THIRD == 1 || THIRD == 2 || THIRD == 4;
    constexpr bool LOAD_B = RULE != CYCLE_FIRST, STORE_B = RULE != CYCLE_REFRESH, USE_M = RULE == CYCLE_REFRESH;
    const uint32_t tid = threadIdx.x;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    double norm_acc = 0.0;
    for (uint32_t t = tile_lo + blockIdx.x; t < tile_hi; t += gridDim.x) {
        const Tile tl = tiles[t];
        const uint32_t tensor = tl.tensor;
        gf32 *th = to_global(theta_tab[tensor]) + tl.start;
        gf32 *mm = USE_M ? to_global(m_tab[tensor]) + tl.start : nullptr;
        gf32 *bb = to_global(buf_tab[tensor]) + tl.start;
        gf32 *ac = THIRD != 0 ? to_global(acc_tab[tensor]) + tl.start : nullptr;
        gf32 *pd = PULL ? to_global(pull_tab[tensor]) + tl.start : nullptr;
        const auto *g = to_global(static_cast<const GT *>(gargs.p[tensor - tensor_base])) + tl.start;
        if (tl.len == TILE_ELEMS) {
            f32x4 gv[UNROLL], bv[UNROLL], mv[UNROLL], tv[UNROLL], av[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t off = (u * BLOCK_THREADS + tid) * VEC;
                gv[u] = grad4<FROM_END, NT>(g, pd, off, gw);
                bv[u] = LOAD_B ? ld4<NT>(bb + off) : zero;
                mv[u] = USE_M ? ld4<NT>(mm + off) : zero;
                tv[u] = ld4<NT>(th + off);
                if constexpr (LOAD_THIRD) av[u] = ld4<NT>(ac + off);
            }
            if constexpr (NORM) {
                float q = 0.f;
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) q = sumsq4(gv[u], q);
                norm_acc += static_cast<double>(q);
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t off = (u * BLOCK_THREADS + tid) * VEC;
                if constexpr (MERGE) {
                    tv[u] = merge4(tv[u], av[u], alpha, keep);
                    av[u] = THIRD == 1 ? zero : tv[u];
                }
                const f32x4 s = delayed_update4<RULE>(tv[u], mv[u], bv[u], gv[u], eta, beta, cgd, inv_d);
                if constexpr (STORE_B) st4<NT>(bb + off, bv[u]);
                if constexpr (USE_M) st4<NT>(mm + off, mv[u]);
                st4<NT>(th + off, tv[u]);
                if constexpr (PULL) st4<NT>(pd + off, tv[u]);
                if constexpr (THIRD == 1) st4<NT>(ac + off, add4(av[u], s));
                if constexpr (THIRD == 2) st4<NT>(ac + off, sub4(av[u], tv[u]));
                if constexpr (THIRD == 3) st4<NT>(ac + off, add4(zero, s));
                if constexpr (THIRD == 4) st4<NT>(ac + off, av[u]);
            }
        } else {
            const uint32_t len = tl.len;
            for (uint32_t off = tid * VEC; off < len; off += BLOCK_THREADS * VEC) {
                if (off + VEC <= len) {
                    f32x4 gv = grad4<FROM_END, NT>(g, pd, off, gw), tv = ld4<NT>(th + off);
                    f32x4 bv = LOAD_B ? ld4<NT>(bb + off) : zero, mv = USE_M ? ld4<NT>(mm + off) : zero;
                    f32x4 av = zero;
                    if constexpr (LOAD_THIRD) av = ld4<NT>(ac + off);
                    if constexpr (NORM) norm_acc += static_cast<double>(sumsq4(gv, 0.f));
                    if constexpr (MERGE) {
                        tv = merge4(tv, av, alpha, keep);
                        av = THIRD == 1 ? zero : tv;
                    }
                    const f32x4 s = delayed_update4<RULE>(tv, mv, bv, gv, eta, beta, cgd, inv_d);
                    if constexpr (STORE_B) st4<NT>(bb + off, bv);
                    if constexpr (USE_M) st4<NT>(mm + off, mv);
                    st4<NT>(th + off, tv);
                    if constexpr (PULL) st4<NT>(pd + off, tv);
                    if constexpr (THIRD == 1) st4<NT>(ac + off, add4(av, s));
                    if constexpr (THIRD == 2) st4<NT>(ac + off, sub4(av, tv));
                    if constexpr (THIRD == 3) st4<NT>(ac + off, add4(zero, s));
                    if constexpr (THIRD == 4) st4<NT>(ac + off, av);
                } else {
                    for (uint32_t k = off; k < len; ++k) {      // ragged tail: fewer than 4 elements
                        float tv = th[k], bv = LOAD_B ? bb[k] : 0.f, mv = USE_M ? mm[k] : 0.f;
                        float av = 0.f;
                        if constexpr (LOAD_THIRD) av = ac[k];
                        const float gk = grad1<FROM_END>(g, pd, k, gw);
                        if constexpr (NORM) norm_acc += static_cast<double>(__fmul_rn(gk, gk));
                        if constexpr (MERGE) {
                            tv = merge1(tv, av, alpha, keep);
                            av = THIRD == 1 ? 0.f : tv;
                        }
                        const float s = delayed_update<RULE>(tv, mv, bv, gk, eta, beta, cgd, inv_d);
                        if constexpr (STORE_B) bb[k] = bv;
                        if constexpr (USE_M) mm[k] = mv;
                        th[k] = tv;
                        if constexpr (PULL) pd[k] = tv;
                        if constexpr (THIRD == 1) ac[k] = __fadd_rn(av, s);
                        if constexpr (THIRD == 2) ac[k] = __fsub_rn(av, tv);
                        if constexpr (THIRD == 3) ac[k] = __fadd_rn(0.f, s);
                        if constexpr (THIRD == 4) ac[k] = av;
                    }
                }
            }
        }
    }
    if constexpr (NORM) block_sum_store(norm_acc, partials + blockIdx.x);
}

// S3 under the delayed rule.  G and out may alias.
template <int RULE>
__global__ void __launch_bounds__(BLOCK_THREADS)
gps_update_delayed_kernel(const Tile *__restrict__ tiles, uint32_t tile_lo, uint32_t tile_hi,
                          float *const *__restrict__ Theta_tab, float *const *__restrict__ M_tab,
                          float *const *__restrict__ buf_tab, float *const *G_tab, float *const *out_tab, float eta,
                          float beta, float cgd, float inv_d) {
    constexpr bool NT = true;
    constexpr bool LOAD_B = RULE != CYCLE_FIRST, STORE_B = RULE != CYCLE_REFRESH, USE_M = RULE == CYCLE_REFRESH;
    const uint32_t tid = threadIdx.x;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    for (uint32_t t = tile_lo + blockIdx.x; t < tile_hi; t += gridDim.x) {
        const Tile tl = tiles[t];
        const uint32_t tensor = tl.tensor;
        gf32 *Th = to_global(Theta_tab[tensor]) + tl.start;
        gf32 *Mm = USE_M ? to_global(M_tab[tensor]) + tl.start : nullptr;
        gf32 *Bb = to_global(buf_tab[tensor]) + tl.start;
        const gf32 *G = to_global(G_tab[tensor]) + tl.start;
        gf32 *out = to_global(out_tab[tensor]) + tl.start;
        if (tl.len == TILE_ELEMS) {
            f32x4 gv[UNROLL], bv[UNROLL], mv[UNROLL], tv[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t off = (u * BLOCK_THREADS + tid) * VEC;
                gv[u] = ld4<NT>(G + off);
                bv[u] = LOAD_B ? ld4<NT>(Bb + off) : zero;
                mv[u] = USE_M ? ld4<NT>(Mm + off) : zero;
                tv[u] = ld4<NT>(Th + off);
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t off = (u * BLOCK_THREADS + tid) * VEC;
                delayed_update4<RULE>(tv[u], mv[u], bv[u], gv[u], eta, beta, cgd, inv_d);
                if constexpr (STORE_B) st4<NT>(Bb + off, bv[u]);
                if constexpr (USE_M) st4<NT>(Mm + off, mv[u]);
                st4<NT>(Th + off, tv[u]);
                st4<NT>(out + off, tv[u]);
            }
        } else {
            const uint32_t len = tl.len;
            for (uint32_t off = tid * VEC; off < len; off += BLOCK_THREADS * VEC) {
                if (off + VEC <= len) {
                    f32x4 gv = ld4<NT>(G + off), tv = ld4<NT>(Th + off);
                    f32x4 bv = LOAD_B ? ld4<NT>(Bb + off) : zero, mv = USE_M ? ld4<NT>(Mm + off) : zero;
                    delayed_update4<RULE>(tv, mv, bv, gv, eta, beta, cgd, inv_d);
                    if constexpr (STORE_B) st4<NT>(Bb + off, bv);
                    if constexpr (USE_M) st4<NT>(Mm + off, mv);
                    st4<NT>(Th + off, tv);
                    st4<NT>(out + off, tv);
                } else {
                    for (uint32_t k = off; k < len; ++k) {
                        float tv = Th[k], bv = LOAD_B ? Bb[k] : 0.f, mv = USE_M ? Mm[k] : 0.f;
                        delayed_update<RULE>(tv, mv, bv, G[k], eta, beta, cgd, inv_d);
                        if constexpr (STORE_B) Bb[k] = bv;
                        if constexpr (USE_M) Mm[k] = mv;
                        Th[k] = tv; out[k] = tv;
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// S4: merge the returned global model into the local model and restart the accumulation.
// With NORM every workgroup also leaves the sum of (theta - Theta_i)^2 before the merge in partials[blockIdx.x].
// OUT says what the third buffer receives: MERGE_CLEAR zeros (the accumulation restarts), MERGE_SNAPSHOT the merged model
// (the new snapshot theta_{t_last}), MERGE_LEAVE nothing -- the first update that accumulates afterwards overwrites it.
template <bool NT, bool NORM, int OUT>
__global__ void __launch_bounds__(BLOCK_THREADS)
lps_merge_kernel(const Tile *__restrict__ tiles, uint32_t tile_lo, uint32_t tile_hi,
                 float *const *__restrict__ theta_tab, float *const *__restrict__ inbox_tab, float alpha, float keep,
                 double *__restrict__ partials) {
    const uint32_t tid = threadIdx.x;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    double norm_acc = 0.0;
    for (uint32_t t = tile_lo + blockIdx.x; t < tile_hi; t += gridDim.x) {
        const Tile tl = tiles[t];
        const uint32_t tensor = tl.tensor;
        gf32 *th = to_global(theta_tab[tensor]) + tl.start;
        gf32 *in = to_global(inbox_tab[tensor]) + tl.start;
        if (tl.len == TILE_ELEMS) {
            f32x4 tv[UNROLL], iv[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t off = (u * BLOCK_THREADS + tid) * VEC;
                tv[u] = ld4<NT>(th + off);
                iv[u] = ld4<NT>(in + off);
            }
            if constexpr (NORM) {
                float q = 0.f;
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) q = sumsq4(sub4(tv[u], iv[u]), q);
                norm_acc += static_cast<double>(q);
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t off = (u * BLOCK_THREADS + tid) * VEC;
                const f32x4 merged = merge4(tv[u], iv[u], alpha, keep);
                st4<NT>(th + off, merged);
                if constexpr (OUT != MERGE_LEAVE) st4<NT>(in + off, OUT == MERGE_SNAPSHOT ? merged : zero);
            }
        } else {
            const uint32_t len = tl.len;
            for (uint32_t off = tid * VEC; off < len; off += BLOCK_THREADS * VEC) {
                if (off + VEC <= len) {
                    const f32x4 tv = ld4<NT>(th + off), iv = ld4<NT>(in + off);
                    if constexpr (NORM) norm_acc += static_cast<double>(sumsq4(sub4(tv, iv), 0.f));
                    const f32x4 merged = merge4(tv, iv, alpha, keep);
                    st4<NT>(th + off, merged);
                    if constexpr (OUT != MERGE_LEAVE) st4<NT>(in + off, OUT == MERGE_SNAPSHOT ? merged : zero);
                } else {
                    for (uint32_t k = off; k < len; ++k) {
                        const float tk = th[k], ik = in[k];
                        if constexpr (NORM) {
                            const float d = __fsub_rn(tk, ik);
                            norm_acc += static_cast<double>(__fmul_rn(d, d));
                        }
                        const float merged = merge1(tk, ik, alpha, keep);
                        th[k] = merged;
                        if constexpr (OUT != MERGE_LEAVE) in[k] = OUT == MERGE_SNAPSHOT ? merged : 0.f;
                    }
                }
            }
        }
    }
    if constexpr (NORM) block_sum_store(norm_acc, partials + blockIdx.x);
}

// Add up the per-workgroup partial sums in a fixed order (one workgroup, fp64): *out = sum(partials[0..n)).
__global__ void __launch_bounds__(BLOCK_THREADS)
norm_finalize_kernel(const double *__restrict__ partials, uint32_t n, double *__restrict__ out) {
    double v = 0.0;
    for (uint32_t i = threadIdx.x; i < n; i += BLOCK_THREADS) v += partials[i];
    block_sum_store(v, out);
}

// ---------------------------------------------------------------------------------------------
// S5: copy a model out.
template <bool NT>
__global__ void __launch_bounds__(BLOCK_THREADS)
pull_kernel(const Tile *__restrict__ tiles, uint32_t tile_lo, uint32_t tile_hi, uint32_t tensor_base,
            float *const *__restrict__ src_tab, PtrArgs dargs) {
    const uint32_t tid = threadIdx.x;
    for (uint32_t t = tile_lo + blockIdx.x; t < tile_hi; t += gridDim.x) {
        const Tile tl = tiles[t];
        const uint32_t tensor = tl.tensor;
        const gf32 *src = to_global(src_tab[tensor]) + tl.start;
        gf32 *dst = to_global(static_cast<float *>(const_cast<void *>(dargs.p[tensor - tensor_base]))) + tl.start;
        if (tl.len == TILE_ELEMS) {
            f32x4 v[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) v[u] = ld4<NT>(src + (u * BLOCK_THREADS + tid) * VEC);
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) st4<NT>(dst + (u * BLOCK_THREADS + tid) * VEC, v[u]);
        } else {
            const uint32_t len = tl.len;
            for (uint32_t off = tid * VEC; off < len; off += BLOCK_THREADS * VEC) {
                if (off + VEC <= len) st4<NT>(dst + off, ld4<NT>(src + off));
                else for (uint32_t k = off; k < len; ++k) dst[k] = src[k];
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Alg. 1, LPS initialisation: theta <- Theta_0, m <- 0, third buffer <- 0 (or <- Theta_0 if it is to hold the snapshot
// theta_{t_last}).  With src_tab == nullptr only m is zero-filled.  MB: the momentum tensors hold bfloat16.
template <bool MB>
__global__ void __launch_bounds__(BLOCK_THREADS)
init_kernel(const Tile *__restrict__ tiles, uint32_t tile_lo, uint32_t tile_hi, float *const *src_tab,
            float *const *theta_tab, float *const *m_tab, float *const *acc_tab, bool snapshot) {
    const uint32_t tid = threadIdx.x;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    for (uint32_t t = tile_lo + blockIdx.x; t < tile_hi; t += gridDim.x) {
        const Tile tl = tiles[t];
        const uint32_t tensor = tl.tensor;
        const uint32_t len = tl.len;
        auto *mm = momentum_ptr<MB>(m_tab[tensor]) + tl.start;
        const gf32 *src = src_tab ? to_global(src_tab[tensor]) + tl.start : nullptr;
        gf32 *th = src_tab ? to_global(theta_tab[tensor]) + tl.start : nullptr;
        gf32 *ac = src_tab ? to_global(acc_tab[tensor]) + tl.start : nullptr;
        for (uint32_t off = tid * VEC; off < len; off += BLOCK_THREADS * VEC) {
            if (off + VEC <= len) {
                stm4<false>(mm + off, zero);
                if (src_tab) {
                    const f32x4 v = ld4<false>(src + off);
                    st4<false>(th + off, v);
                    st4<false>(ac + off, snapshot ? v : zero);
                }
            } else {
                for (uint32_t k = off; k < len; ++k) {
                    stm1(mm + k, 0.f);
                    if (src_tab) { th[k] = src[k]; ac[k] = snapshot ? src[k] : 0.f; }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Placement probe: read two buffers and write both back unchanged, tile by tile.  Only its duration
// matters: two buffers served by the same HBM region sweep measurably slower than two served by
// different regions.
__global__ void __launch_bounds__(BLOCK_THREADS)
probe_pair_kernel(float *a, float *b, uint32_t n_tiles) {
    const uint32_t tid = threadIdx.x;
    gf32 *ga = to_global(a), *gb = to_global(b);
    for (uint32_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const size_t base = static_cast<size_t>(t) * TILE_ELEMS;
        f32x4 va[UNROLL], vb[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const size_t off = base + (u * BLOCK_THREADS + tid) * VEC;
            va[u] = ld4<true>(ga + off);
            vb[u] = ld4<true>(gb + off);
        }
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const size_t off = base + (u * BLOCK_THREADS + tid) * VEC;
            // The values go back unchanged, but the compiler must not know that, or it would drop the
            // stores (and then the loads) as redundant: pass them through an empty asm statement.
            asm volatile("" : "+v"(va[u]), "+v"(vb[u]));
            st4<true>(ga + off, va[u]);
            st4<true>(gb + off, vb[u]);
        }
    }
}

__global__ void __launch_bounds__(BLOCK_THREADS)
store_pointers_kernel(float **table, PtrArgs src, uint32_t first, uint32_t count) {
    for (uint32_t i = threadIdx.x; i < count; i += BLOCK_THREADS)
        table[first + i] = static_cast<float *>(const_cast<void *>(src.p[i]));
}

// Streaming probe: read NR buffers and write NW others, tile by tile with the access pattern of the update kernels
// (UNR 128-bit non-temporal accesses per thread and stream, all loads of a tile issued before anything else).
// No arithmetic; loaded values are only "used" by an empty asm statement so the loads stay, stores write `fill`.
template <int NR, int NW, int UNR>
__global__ void __launch_bounds__(BLOCK_THREADS)
probe_streams_kernel(ProbeArgs a, uint32_t n_tiles, float fill) {
    const uint32_t tid = threadIdx.x;
    const f32x4 fv = {fill, fill, fill, fill};
    constexpr size_t TILE = (size_t)BLOCK_THREADS * VEC * UNR;
    for (uint32_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        const size_t base = static_cast<size_t>(t) * TILE;
        f32x4 v[NR > 0 ? NR : 1][UNR];
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int u = 0; u < UNR; ++u)
                v[r][u] = ld4<true>(to_global(a.rd[r]) + base + (u * BLOCK_THREADS + tid) * VEC);
#pragma unroll
        for (int r = 0; r < NR; ++r)
#pragma unroll
            for (int u = 0; u < UNR; ++u) asm volatile("" : : "v"(v[r][u]));
#pragma unroll
        for (int w = 0; w < NW; ++w)
#pragma unroll
            for (int u = 0; u < UNR; ++u)
                st4<true>(to_global(a.wr[w]) + base + (u * BLOCK_THREADS + tid) * VEC, fv);
    }
}

// Partial sums of the norm monitors for the entry point that allocates nothing.  In host code this name is only a
// handle for hipGetSymbolAddress; kernels receive the address that call returns.
static __device__ __align__(256) double scratch[STATIC_SCRATCH_DOUBLES];

inline dim3 grid_for(TileRange r, LaunchShape shape) {
    uint32_t n = r.hi - r.lo;
    uint32_t cap = shape.grid_cap > 0 ? (uint32_t)shape.grid_cap : 1u;
    return dim3(n < cap ? n : cap);
}

}  // namespace

hipError_t static_scratch(double **ptr) {
    constexpr int MAX_DEVICES = 64;
    static std::atomic<double *> per_device[MAX_DEVICES];      // zero-initialised: "not looked up yet"
    *ptr = nullptr;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    double *p = per_device[dev].load(std::memory_order_acquire);
    if (!p) {
        void *sym = nullptr;
        e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));     // this device's copy of the array
        if (e != hipSuccess) return e;
        if (!sym) return hipErrorInvalidSymbol;
        p = static_cast<double *>(sym);
        per_device[dev].store(p, std::memory_order_release);
    }
    *ptr = p;
    return hipSuccess;
}

uint32_t launch_grid_size(TileRange r, LaunchShape shape) { return r.hi > r.lo ? grid_for(r, shape).x : 0u; }

hipError_t launch_lps_update(hipStream_t stream, const Tile *tiles, TileRange r, float *const *theta, float *const *m,
                             float *const *acc, float *const *pull, const PtrArgs &g, int g_kind, int third_mode,
                             float eta, float beta, float cg, float gw, double *norm_partials, LaunchShape shape,
                             bool m_bf16) {
    if (r.hi <= r.lo) return hipSuccess;
    if (g_kind < GRAD_F32 || g_kind > GRAD_F16 || third_mode < THIRD_NONE || third_mode > THIRD_RESTART ||
        (g_kind == GRAD_END_MODEL && !pull))
        return hipErrorInvalidValue;
    const dim3 grid = grid_for(r, shape), block(BLOCK_THREADS);
#define HALOS_LAUNCH_UPD_MB(GT, THIRD, NT, PULL, END, MB)                                                                 \
    do {                                                                                                                 \
        if (norm_partials)                                                                                               \
            lps_update_kernel<GT, THIRD, NT, PULL, true, END, MB><<<grid, block, 0, stream>>>(                           \
                tiles, r.lo, r.hi, r.tensor_base, theta, m, acc, pull, g, eta, beta, cg, gw, norm_partials);             \
        else                                                                                                             \
            lps_update_kernel<GT, THIRD, NT, PULL, false, END, MB><<<grid, block, 0, stream>>>(                          \
                tiles, r.lo, r.hi, r.tensor_base, theta, m, acc, pull, g, eta, beta, cg, gw, nullptr);                   \
    } while (0)
#define HALOS_LAUNCH_UPD(GT, THIRD, NT, PULL, END) \
    do { if (m_bf16) HALOS_LAUNCH_UPD_MB(GT, THIRD, NT, PULL, END, true); else HALOS_LAUNCH_UPD_MB(GT, THIRD, NT, PULL, END, false); } while (0)
#define HALOS_LAUNCH_UPD_NT(GT, THIRD, PULL, END) \
    do { if (shape.nontemporal) HALOS_LAUNCH_UPD(GT, THIRD, true, PULL, END); else HALOS_LAUNCH_UPD(GT, THIRD, false, PULL, END); } while (0)
#define HALOS_LAUNCH_UPD_THIRD(GT, PULL, END)                                  \
    do {                                                                       \
        if (third_mode == THIRD_NONE) HALOS_LAUNCH_UPD_NT(GT, 0, PULL, END);   \
        else if (third_mode == THIRD_ADD) HALOS_LAUNCH_UPD_NT(GT, 1, PULL, END); \
        else if (third_mode == THIRD_FREEZE_SNAPSHOT) HALOS_LAUNCH_UPD_NT(GT, 2, PULL, END); \
        else HALOS_LAUNCH_UPD_NT(GT, 3, PULL, END);                            \
    } while (0)
#define HALOS_LAUNCH_UPD_PULL(GT) \
    do { if (pull) HALOS_LAUNCH_UPD_THIRD(GT, true, false); else HALOS_LAUNCH_UPD_THIRD(GT, false, false); } while (0)
    if (g_kind == GRAD_END_MODEL) HALOS_LAUNCH_UPD_THIRD(float, true, true);
    else if (g_kind == GRAD_BF16) HALOS_LAUNCH_UPD_PULL(unsigned short);
    else if (g_kind == GRAD_F16) HALOS_LAUNCH_UPD_PULL(_Float16);
    else HALOS_LAUNCH_UPD_PULL(float);
#undef HALOS_LAUNCH_UPD_PULL
#undef HALOS_LAUNCH_UPD_THIRD
#undef HALOS_LAUNCH_UPD_NT
#undef HALOS_LAUNCH_UPD
#undef HALOS_LAUNCH_UPD_MB
    return hipGetLastError();
}

hipError_t launch_lps_update_multi(hipStream_t stream, const Tile *tiles, TileRange r, float *const *theta, float *const *m,
                                   float *const *acc, const MultiArgs &a, bool average, int g_kind, int third_mode,
                                   float eta, float beta, float cg, float inv_n, LaunchShape shape, bool m_bf16) {
    if (r.hi <= r.lo) return hipSuccess;
    if (a.n_in < 1 || a.n_in > MAX_MULTI || a.n_acc < 0 || a.n_acc > a.n_in || third_mode < THIRD_NONE ||
        third_mode > THIRD_RESTART || (g_kind != GRAD_F32 && g_kind != GRAD_BF16 && g_kind != GRAD_F16))
        return hipErrorInvalidValue;
    if (a.merge && (average || (third_mode != THIRD_ADD && third_mode != THIRD_FREEZE_SNAPSHOT))) return hipErrorInvalidValue;
    bool pull = false;
    for (int i = 0; i < a.n_in; ++i) {
        if (!a.delta[i]) return hipErrorInvalidValue;
        pull = pull || a.pull[i] != nullptr;
    }
    const dim3 grid = grid_for(r, shape), block(BLOCK_THREADS);
#define HALOS_LAUNCH_MULTI(GT, SEQ, THIRD, PULL)                                                                                      \
    do {                                                                                                                             \
        if (m_bf16)                                                                                                                  \
            lps_update_multi_kernel<GT, SEQ, THIRD, PULL, true><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, theta, m, acc, a, eta, beta, cg, inv_n); \
        else                                                                                                                         \
            lps_update_multi_kernel<GT, SEQ, THIRD, PULL, false><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, theta, m, acc, a, eta, beta, cg, inv_n); \
    } while (0)
#define HALOS_LAUNCH_MULTI_THIRD(GT, SEQ, PULL)                                    \
    do {                                                                           \
        if (third_mode == THIRD_NONE) HALOS_LAUNCH_MULTI(GT, SEQ, 0, PULL);        \
        else if (third_mode == THIRD_ADD) HALOS_LAUNCH_MULTI(GT, SEQ, 1, PULL);    \
        else if (third_mode == THIRD_FREEZE_SNAPSHOT) HALOS_LAUNCH_MULTI(GT, SEQ, 2, PULL); \
        else HALOS_LAUNCH_MULTI(GT, SEQ, 3, PULL);                                 \
    } while (0)
#define HALOS_LAUNCH_MULTI_MERGE(GT, THIRD, PULL)                                                                                     \
    do {                                                                                                                             \
        if (m_bf16)                                                                                                                  \
            lps_update_multi_kernel<GT, true, THIRD, PULL, true, true><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, theta, m, acc, a, eta, beta, cg, inv_n); \
        else                                                                                                                         \
            lps_update_multi_kernel<GT, true, THIRD, PULL, false, true><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, theta, m, acc, a, eta, beta, cg, inv_n); \
    } while (0)
#define HALOS_LAUNCH_MULTI_KIND(GT)                                                \
    do {                                                                           \
        if (a.merge) {                                                             \
            if (third_mode == THIRD_ADD) { if (pull) HALOS_LAUNCH_MULTI_MERGE(GT, 1, true); else HALOS_LAUNCH_MULTI_MERGE(GT, 1, false); } \
            else { if (pull) HALOS_LAUNCH_MULTI_MERGE(GT, 2, true); else HALOS_LAUNCH_MULTI_MERGE(GT, 2, false); } \
        }                                                                          \
        else if (average) HALOS_LAUNCH_MULTI_THIRD(GT, false, false);              \
        else if (pull) HALOS_LAUNCH_MULTI_THIRD(GT, true, true);                   \
        else HALOS_LAUNCH_MULTI_THIRD(GT, true, false);                            \
    } while (0)
    if (g_kind == GRAD_BF16) HALOS_LAUNCH_MULTI_KIND(unsigned short);
    else if (g_kind == GRAD_F16) HALOS_LAUNCH_MULTI_KIND(_Float16);
    else HALOS_LAUNCH_MULTI_KIND(float);
#undef HALOS_LAUNCH_MULTI_KIND
#undef HALOS_LAUNCH_MULTI_MERGE
#undef HALOS_LAUNCH_MULTI_THIRD
#undef HALOS_LAUNCH_MULTI
    return hipGetLastError();
}

hipError_t launch_gps_update(hipStream_t stream, const Tile *tiles, TileRange r, float *const *Theta, float *const *M,
                             float *const *G, float *const *out, float eta, float beta, float cg, LaunchShape shape,
                             bool m_bf16) {
    if (r.hi <= r.lo) return hipSuccess;
    const dim3 grid = grid_for(r, shape), block(BLOCK_THREADS);
    if (shape.nontemporal) {
        if (m_bf16) gps_update_kernel<true, true><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, Theta, M, G, out, eta, beta, cg);
        else gps_update_kernel<true, false><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, Theta, M, G, out, eta, beta, cg);
    } else {
        if (m_bf16) gps_update_kernel<false, true><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, Theta, M, G, out, eta, beta, cg);
        else gps_update_kernel<false, false><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, Theta, M, G, out, eta, beta, cg);
    }
    return hipGetLastError();
}

hipError_t launch_gps_update_nomom(hipStream_t stream, const Tile *tiles, TileRange r, float *const *Theta,
                                   float *const *G, float *const *out, float eta, float cg, LaunchShape shape) {
    if (r.hi <= r.lo) return hipSuccess;
    const dim3 grid = grid_for(r, shape), block(BLOCK_THREADS);
    if (shape.nontemporal)
        gps_update_nomom_kernel<true><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, Theta, G, out, eta, cg);
    else
        gps_update_nomom_kernel<false><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, Theta, G, out, eta, cg);
    return hipGetLastError();
}

hipError_t launch_lps_update_delayed(hipStream_t stream, const Tile *tiles, TileRange r, float *const *theta,
                                     float *const *m, float *const *buffer, float *const *acc, float *const *pull,
                                     const PtrArgs &g, int g_kind, int third_mode, int cycle_pos, float eta,
                                     float beta, float cgd, float inv_d, float gw, double *norm_partials, LaunchShape shape,
                                     bool merge, float alpha, float keep) {
    if (r.hi <= r.lo) return hipSuccess;
    if (cycle_pos < CYCLE_FIRST || cycle_pos > CYCLE_REFRESH || third_mode < THIRD_NONE ||
        third_mode > (merge ? THIRD_MERGED_SNAPSHOT : THIRD_RESTART) ||
        g_kind < GRAD_F32 || g_kind > GRAD_F16 || (g_kind == GRAD_END_MODEL && !pull))
        return hipErrorInvalidValue;
    const dim3 grid = grid_for(r, shape), block(BLOCK_THREADS);
    if (merge) {        // merge-first pass: plain deltas with the model handed back, no monitors
        if (!pull || norm_partials || g_kind == GRAD_END_MODEL ||
            (third_mode != THIRD_ADD && third_mode != THIRD_FREEZE_SNAPSHOT && third_mode != THIRD_MERGED_SNAPSHOT))
            return hipErrorInvalidValue;
#define HALOS_LAUNCH_DNM(GT, THIRD, RULE)                                                                               \
    lps_update_delayed_kernel<GT, THIRD, true, RULE, false, false, true><<<grid, block, 0, stream>>>(                   \
        tiles, r.lo, r.hi, r.tensor_base, theta, m, buffer, acc, pull, g, eta, beta, cgd, inv_d, gw, nullptr, alpha, keep)
#define HALOS_LAUNCH_DNM_RULE(GT, THIRD)                                                 \
    do {                                                                                 \
        if (cycle_pos == CYCLE_FIRST) HALOS_LAUNCH_DNM(GT, THIRD, CYCLE_FIRST);          \
        else if (cycle_pos == CYCLE_INNER) HALOS_LAUNCH_DNM(GT, THIRD, CYCLE_INNER);     \
        else HALOS_LAUNCH_DNM(GT, THIRD, CYCLE_REFRESH);                                 \
    } while (0)
#define HALOS_LAUNCH_DNM_THIRD(GT)                                                       \
    do {                                                                                 \
        if (third_mode == THIRD_ADD) HALOS_LAUNCH_DNM_RULE(GT, 1);                       \
        else if (third_mode == THIRD_FREEZE_SNAPSHOT) HALOS_LAUNCH_DNM_RULE(GT, 2);      \
        else HALOS_LAUNCH_DNM_RULE(GT, 4);                                               \
    } while (0)
        if (g_kind == GRAD_BF16) HALOS_LAUNCH_DNM_THIRD(unsigned short);
        else if (g_kind == GRAD_F16) HALOS_LAUNCH_DNM_THIRD(_Float16);
        else HALOS_LAUNCH_DNM_THIRD(float);
#undef HALOS_LAUNCH_DNM_THIRD
#undef HALOS_LAUNCH_DNM_RULE
#undef HALOS_LAUNCH_DNM
        return hipGetLastError();
    }
#define HALOS_LAUNCH_DN(GT, THIRD, PULL, RULE, END)                                                                     \
    do {                                                                                                                \
        if (norm_partials)                                                                                              \
            lps_update_delayed_kernel<GT, THIRD, PULL, RULE, END, true><<<grid, block, 0, stream>>>(                    \
                tiles, r.lo, r.hi, r.tensor_base, theta, m, buffer, acc, pull, g, eta, beta, cgd, inv_d, gw, norm_partials, 0.f, 0.f); \
        else                                                                                                            \
            lps_update_delayed_kernel<GT, THIRD, PULL, RULE, END, false><<<grid, block, 0, stream>>>(                   \
                tiles, r.lo, r.hi, r.tensor_base, theta, m, buffer, acc, pull, g, eta, beta, cgd, inv_d, gw, nullptr, 0.f, 0.f); \
    } while (0)
#define HALOS_LAUNCH_DN_RULE(GT, THIRD, PULL, END)                                       \
    do {                                                                                 \
        if (cycle_pos == CYCLE_FIRST) HALOS_LAUNCH_DN(GT, THIRD, PULL, CYCLE_FIRST, END); \
        else if (cycle_pos == CYCLE_INNER) HALOS_LAUNCH_DN(GT, THIRD, PULL, CYCLE_INNER, END); \
        else HALOS_LAUNCH_DN(GT, THIRD, PULL, CYCLE_REFRESH, END);                       \
    } while (0)
#define HALOS_LAUNCH_DN_THIRD(GT, PULL, END)                                   \
    do {                                                                       \
        if (third_mode == THIRD_NONE) HALOS_LAUNCH_DN_RULE(GT, 0, PULL, END);  \
        else if (third_mode == THIRD_ADD) HALOS_LAUNCH_DN_RULE(GT, 1, PULL, END); \
        else if (third_mode == THIRD_FREEZE_SNAPSHOT) HALOS_LAUNCH_DN_RULE(GT, 2, PULL, END); \
        else HALOS_LAUNCH_DN_RULE(GT, 3, PULL, END);                           \
    } while (0)
#define HALOS_LAUNCH_DN_PULL(GT) \
    do { if (pull) HALOS_LAUNCH_DN_THIRD(GT, true, false); else HALOS_LAUNCH_DN_THIRD(GT, false, false); } while (0)
    if (g_kind == GRAD_END_MODEL) HALOS_LAUNCH_DN_THIRD(float, true, true);
    else if (g_kind == GRAD_BF16) HALOS_LAUNCH_DN_PULL(unsigned short);
    else if (g_kind == GRAD_F16) HALOS_LAUNCH_DN_PULL(_Float16);
    else HALOS_LAUNCH_DN_PULL(float);
#undef HALOS_LAUNCH_DN_PULL
#undef HALOS_LAUNCH_DN_THIRD
#undef HALOS_LAUNCH_DN_RULE
#undef HALOS_LAUNCH_DN
    return hipGetLastError();
}

hipError_t launch_gps_update_delayed(hipStream_t stream, const Tile *tiles, TileRange r, float *const *Theta,
                                     float *const *M, float *const *buffer, float *const *G, float *const *out,
                                     int cycle_pos, float eta, float beta, float cgd, float inv_d, LaunchShape shape) {
    if (r.hi <= r.lo) return hipSuccess;
    if (cycle_pos < CYCLE_FIRST || cycle_pos > CYCLE_REFRESH) return hipErrorInvalidValue;
    const dim3 grid = grid_for(r, shape), block(BLOCK_THREADS);
    if (cycle_pos == CYCLE_FIRST)
        gps_update_delayed_kernel<CYCLE_FIRST><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, Theta, M, buffer, G, out, eta, beta, cgd, inv_d);
    else if (cycle_pos == CYCLE_INNER)
        gps_update_delayed_kernel<CYCLE_INNER><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, Theta, M, buffer, G, out, eta, beta, cgd, inv_d);
    else
        gps_update_delayed_kernel<CYCLE_REFRESH><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, Theta, M, buffer, G, out, eta, beta, cgd, inv_d);
    return hipGetLastError();
}

hipError_t launch_lps_merge(hipStream_t stream, const Tile *tiles, TileRange r, float *const *theta,
                            float *const *inbox, float alpha, float keep, int third_out, double *norm_partials,
                            LaunchShape shape) {
    if (r.hi <= r.lo) return hipSuccess;
    if (third_out < MERGE_CLEAR || third_out > MERGE_LEAVE) return hipErrorInvalidValue;
    const dim3 grid = grid_for(r, shape), block(BLOCK_THREADS);
#define HALOS_LAUNCH_MERGE(NT, NORM, OUT) \
    lps_merge_kernel<NT, NORM, OUT><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, theta, inbox, alpha, keep, norm_partials)
#define HALOS_LAUNCH_MERGE_OUT(NT, NORM)                                              \
    do {                                                                              \
        if (third_out == MERGE_CLEAR) HALOS_LAUNCH_MERGE(NT, NORM, MERGE_CLEAR);      \
        else if (third_out == MERGE_SNAPSHOT) HALOS_LAUNCH_MERGE(NT, NORM, MERGE_SNAPSHOT); \
        else HALOS_LAUNCH_MERGE(NT, NORM, MERGE_LEAVE);                               \
    } while (0)
    if (shape.nontemporal) { if (norm_partials) HALOS_LAUNCH_MERGE_OUT(true, true); else HALOS_LAUNCH_MERGE_OUT(true, false); }
    else { if (norm_partials) HALOS_LAUNCH_MERGE_OUT(false, true); else HALOS_LAUNCH_MERGE_OUT(false, false); }
#undef HALOS_LAUNCH_MERGE_OUT
#undef HALOS_LAUNCH_MERGE
    return hipGetLastError();
}

hipError_t launch_norm_finalize(hipStream_t stream, const double *partials, uint32_t n, double *out) {
    norm_finalize_kernel<<<dim3(1), dim3(BLOCK_THREADS), 0, stream>>>(partials, n, out);
    return hipGetLastError();
}

hipError_t launch_pull(hipStream_t stream, const Tile *tiles, TileRange r, float *const *src, const PtrArgs &dst,
                       LaunchShape shape) {
    if (r.hi <= r.lo) return hipSuccess;
    const dim3 grid = grid_for(r, shape), block(BLOCK_THREADS);
    if (shape.nontemporal)
        pull_kernel<true><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, r.tensor_base, src, dst);
    else
        pull_kernel<false><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, r.tensor_base, src, dst);
    return hipGetLastError();
}

hipError_t launch_store_pointers(hipStream_t stream, float **table, const PtrArgs &src, uint32_t first, uint32_t count) {
    if (count == 0) return hipSuccess;
    if (count > (uint32_t)MAX_ARG_TENSORS) return hipErrorInvalidValue;
    store_pointers_kernel<<<dim3(1), dim3(BLOCK_THREADS), 0, stream>>>(table, src, first, count);
    return hipGetLastError();
}

hipError_t launch_init(hipStream_t stream, const Tile *tiles, TileRange r, float *const *src, float *const *theta,
                       float *const *m, float *const *acc, bool snapshot, LaunchShape shape, bool m_bf16) {
    if (r.hi <= r.lo) return hipSuccess;
    const dim3 grid = grid_for(r, shape), block(BLOCK_THREADS);
    if (m_bf16) init_kernel<true><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, src, theta, m, acc, snapshot);
    else init_kernel<false><<<grid, block, 0, stream>>>(tiles, r.lo, r.hi, src, theta, m, acc, snapshot);
    return hipGetLastError();
}

hipError_t launch_probe_pair(hipStream_t stream, float *a, float *b, uint32_t n_tiles, LaunchShape shape) {
    if (n_tiles == 0) return hipSuccess;
    const uint32_t cap = shape.grid_cap > 0 ? (uint32_t)shape.grid_cap : 1u;
    probe_pair_kernel<<<dim3(n_tiles < cap ? n_tiles : cap), dim3(BLOCK_THREADS), 0, stream>>>(a, b, n_tiles);
    return hipGetLastError();
}

namespace {
template <int NR, int NW>
void probe_dispatch_unroll(hipStream_t stream, dim3 grid, const ProbeArgs &a, int unroll, uint32_t n_tiles) {
    const dim3 block(BLOCK_THREADS);
    switch (unroll) {
        case 1: probe_streams_kernel<NR, NW, 1><<<grid, block, 0, stream>>>(a, n_tiles, 0.0f); break;
        case 2: probe_streams_kernel<NR, NW, 2><<<grid, block, 0, stream>>>(a, n_tiles, 0.0f); break;
        case 4: probe_streams_kernel<NR, NW, 4><<<grid, block, 0, stream>>>(a, n_tiles, 0.0f); break;
        case 8: probe_streams_kernel<NR, NW, 8><<<grid, block, 0, stream>>>(a, n_tiles, 0.0f); break;
        default: probe_streams_kernel<NR, NW, 16><<<grid, block, 0, stream>>>(a, n_tiles, 0.0f); break;
    }
}
template <int NR>
void probe_dispatch_writes(hipStream_t stream, dim3 grid, const ProbeArgs &a, int n_write, int unroll, uint32_t n_tiles) {
    switch (n_write) {
        case 0: if constexpr (NR > 0) probe_dispatch_unroll<NR, 0>(stream, grid, a, unroll, n_tiles); break;
        case 1: probe_dispatch_unroll<NR, 1>(stream, grid, a, unroll, n_tiles); break;
        case 2: probe_dispatch_unroll<NR, 2>(stream, grid, a, unroll, n_tiles); break;
        case 3: probe_dispatch_unroll<NR, 3>(stream, grid, a, unroll, n_tiles); break;
        default: probe_dispatch_unroll<NR, 4>(stream, grid, a, unroll, n_tiles); break;
    }
}
}  // namespace

hipError_t launch_probe_streams(hipStream_t stream, const ProbeArgs &a, int n_read, int n_write, int unroll,
                                uint32_t n_tiles, LaunchShape shape) {
    if (n_tiles == 0) return hipSuccess;
    if (n_read < 0 || n_read > MAX_PROBE_STREAMS || n_write < 0 || n_write > MAX_PROBE_STREAMS || n_read + n_write == 0)
        return hipErrorInvalidValue;
    if (unroll != 1 && unroll != 2 && unroll != 4 && unroll != 8 && unroll != 16) return hipErrorInvalidValue;
    const uint32_t cap = shape.grid_cap > 0 ? (uint32_t)shape.grid_cap : 1u;
    const dim3 grid(n_tiles < cap ? n_tiles : cap);
    switch (n_read) {
        case 0: probe_dispatch_writes<0>(stream, grid, a, n_write, unroll, n_tiles); break;
        case 1: probe_dispatch_writes<1>(stream, grid, a, n_write, unroll, n_tiles); break;
        case 2: probe_dispatch_writes<2>(stream, grid, a, n_write, unroll, n_tiles); break;
        case 3: probe_dispatch_writes<3>(stream, grid, a, n_write, unroll, n_tiles); break;
        default: probe_dispatch_writes<4>(stream, grid, a, n_write, unroll, n_tiles); break;
    }
    return hipGetLastError();
}

}  // namespace halos
