// Device-side helpers shared by the row and column kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fm.h"

#include <type_traits>

template <int VEC>
__device__ __forceinline__ void fm_load_vec(const float* __restrict__ p, float (&v)[VEC])
{
    if constexpr (VEC == 4) {
        const float4 t = *reinterpret_cast<const float4*>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else if constexpr (VEC == 2) {
        const float2 t = *reinterpret_cast<const float2*>(p);
        v[0] = t.x; v[1] = t.y;
    } else {
        v[0] = *p;
    }
}

// The same from a row stored as IEEE half precision (the internal copy of V that a pass with
// fm_params.half_gather reads): half the bytes per gathered row, widened to fp32 on arrival.
typedef _Float16 fm_h4 __attribute__((ext_vector_type(4)));
typedef _Float16 fm_h2 __attribute__((ext_vector_type(2)));
template <int VEC>
__device__ __forceinline__ void fm_load_vec(const _Float16* __restrict__ p, float (&v)[VEC])
{
    if constexpr (VEC == 4) {
        const fm_h4 t = *reinterpret_cast<const fm_h4*>(p);
        v[0] = (float)t.x; v[1] = (float)t.y; v[2] = (float)t.z; v[3] = (float)t.w;
    } else if constexpr (VEC == 2) {
        const fm_h2 t = *reinterpret_cast<const fm_h2*>(p);
        v[0] = (float)t.x; v[1] = (float)t.y;
    } else {
        v[0] = (float)*p;
    }
}

// Same load with the non-temporal hint: the line is not kept in L2 ahead of lines that
// were loaded normally.  Used on the column side for rows that will not be gathered again
// soon, so that they do not push a panel's rows out of the 4 MB L2 of the XCD.
typedef float fm_v4f __attribute__((ext_vector_type(4)));
typedef float fm_v2f __attribute__((ext_vector_type(2)));
template <int VEC>
__device__ __forceinline__ void fm_load_vec_nt(const float* __restrict__ p, float (&v)[VEC])
{
    if constexpr (VEC == 4) {
        const fm_v4f t = __builtin_nontemporal_load(reinterpret_cast<const fm_v4f*>(p));
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else if constexpr (VEC == 2) {
        const fm_v2f t = __builtin_nontemporal_load(reinterpret_cast<const fm_v2f*>(p));
        v[0] = t.x; v[1] = t.y;
    } else {
        v[0] = __builtin_nontemporal_load(p);
    }
}

template <int VEC>
__device__ __forceinline__ void fm_store_vec(float* __restrict__ p, const float (&v)[VEC])
{
    if constexpr (VEC == 4) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    } else if constexpr (VEC == 2) {
        *reinterpret_cast<float2*>(p) = make_float2(v[0], v[1]);
    } else {
        *p = v[0];
    }
}

// Sum over the L lanes of a group (L a power of two, groups aligned to L lanes);
// every lane of the group receives the total.  Fixed butterfly order.
template <int L, typename T>
__device__ __forceinline__ T fm_group_sum(T v)
{
#pragma unroll
    for (int o = L / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, L);
    return v;
}

// Sum over all 64 lanes of the wave, fixed butterfly order.
template <typename T>
__device__ __forceinline__ T fm_wave_sum(T v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Loss value and multiplier for one example (cases after eq. updates_v; the loss
// constants make the printed multiplier the exact derivative).  expf only ever sees
// a non-positive argument.
__device__ __forceinline__ void loss_and_multiplier(int32_t loss, float s, float yh, float y, float& l, float& r)
{
    if (loss == FM_LOSS_SQUARED) {
        const float d = yh - y;
        l = 0.5f * d * d;
        r = s * d;
    } else {
        const float mg = y * yh;
        if (mg > 0.f) {
            const float e = expf(-mg);
            l = log1pf(e);
            r = -s * y * e / (1.f + e);
        } else {
            const float e = expf(mg);
            l = -mg + log1pf(e);
            r = -s * y / (1.f + e);
        }
    }
}

// Block b of the floor split of n items into P blocks that holds index i:
// b = floor(((i+1) P - 1) / n)   (inverse of the bound floor(b n / P)).
__device__ __forceinline__ int32_t fm_block_of(int64_t i, int64_t n, int32_t P)
{
    return (int32_t)(((i + 1) * (int64_t)P - 1) / n);
}

// Compile-time loop: f(std::integral_constant<int, I>) for I = 0..N-1.
template <int I, int N, class F>
__device__ __forceinline__ void fm_static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        fm_static_for<I + 1, N>(f);
    }
}

// Value of `v` held by lane T of the caller's L-lane group, T known at compile time:
// a DPP quad permute for groups of up to four lanes (no LDS traffic), the LDS crossbar
// (ds_bpermute) for wider groups.
template <int L, int T>
__device__ __forceinline__ int fm_bcast_i(int v)
{
    if constexpr (L == 1) {
        return v;
    } else if constexpr (L == 2) {
        return __builtin_amdgcn_mov_dpp(v, T == 0 ? 0xA0 : 0xF5, 0xf, 0xf, true);
    } else if constexpr (L == 4) {
        return __builtin_amdgcn_mov_dpp(v, T * 0x55, 0xf, 0xf, true);
    } else if constexpr (L == 8) {
        // two DPP moves instead of a trip through the LDS crossbar: every quad broadcasts its lane
        // T % 4, then the quad that does not hold lane T takes the other quad's value (a row shift by
        // four lanes, written only to the banks of those quads)
        const int x = __builtin_amdgcn_mov_dpp(v, (T % 4) * 0x55, 0xf, 0xf, true);
        if constexpr (T < 4)
            return __builtin_amdgcn_update_dpp(x, x, 0x114 /* row_shr:4 */, 0xf, 0xa, false);
        else
            return __builtin_amdgcn_update_dpp(x, x, 0x104 /* row_shl:4 */, 0xf, 0x5, false);
    } else {
        return __shfl(v, T, L);
    }
}
template <int L, int T>
__device__ __forceinline__ float fm_bcast_f(float v)
{
    return __int_as_float(fm_bcast_i<L, T>(__float_as_int(v)));
}

// Entry slots per lane and iteration so that a group keeps 16 row gathers in flight.
template <int L>
struct FmChunk {
    static constexpr int CH = (16 / L) > 0 ? (16 / L) : 1;
};

// S entry slots (slot s = entry s%L of lane-slot s/L): broadcast each entry's index and
// multiplier inside the group, gather the rows with at most 16 loads in flight, then
// accumulate.
template <int VEC, int L, bool SQ, int S, class IX, class MU, class SRC>
__device__ __forceinline__ void fm_gather_slots(const IX& ix, const MU& mu, const SRC* __restrict__ src,
                                                int64_t stride, int kb, float (&acc)[VEC], float& sq)
{
    constexpr int B = S < 16 ? S : 16;
    fm_static_for<0, S / B>([&](auto bc) {
        constexpr int B0 = decltype(bc)::value * B;
        float g[B][VEC];
        float mt[B];
        fm_static_for<0, B>([&](auto sc) {
            constexpr int s = B0 + decltype(sc)::value;
            constexpr int u = s / L, T = s % L;
            const int raw = fm_bcast_i<L, T>(ix[u]);
            mt[s - B0] = fm_bcast_f<L, T>(mu[u]);
            fm_load_vec<VEC>(src + (int64_t)raw * stride + kb, g[s - B0]);
        });
#pragma unroll
        for (int s = 0; s < B; ++s) {
#pragma unroll
            for (int z = 0; z < VEC; ++z) {
                acc[z] += mt[s] * g[s][z];
                if constexpr (SQ) sq += (mt[s] * mt[s]) * (g[s][z] * g[s][z]);
            }
        }
    });
}

// The common inner loop of the row and the column kernels.  A group of L lanes walks
// the entries [beg,end) of one sparse row (or column): idx[e] names a row of `src`
// (`stride` floats apart) and val[e] its coefficient.  Lane `sub` of the group
//   * loads entry e+sub of every L-entry slot (coalesced) and calls
//       m = own(index, value)      -- per-entry work of that lane, linear in the value;
//                                     returns the multiplier of the gathered row
//   * receives every entry's (index, m) by broadcast and accumulates
//       acc[z] += m * src[index*stride + kb + z]     (and, if SQ, sq += m^2 * src[..]^2).
// Full chunks of L*CH entries run without masking; the tail runs in L-entry slots whose
// missing entries repeat the last entry with value 0.  `kb` must be a valid offset for
// every lane (idle lanes pass 0 and discard acc).
template <int VEC, int L, bool SQ, int CH = FmChunk<L>::CH, class Own, class SRC = float>
__device__ __forceinline__ void fm_gather_accumulate(const int32_t* __restrict__ idx, const float* __restrict__ val,
                                                     int64_t beg, int64_t end, const SRC* __restrict__ src,
                                                     int64_t stride, int sub, int kb, float (&acc)[VEC], float& sq,
                                                     Own&& own)
{
    int64_t e = beg;
    // the lean form (CH == 1) of wide groups takes every entry through the four-at-a-time loop below:
    // few registers, so that more rows or columns are in flight
    constexpr bool CHUNKS = !(CH == 1 && L >= 16);
    for (; CHUNKS && e + L * CH <= end; e += L * CH) {
        int ix[CH];
        float mu[CH];
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int64_t my = e + u * L + sub;
            ix[u] = idx[my];
            mu[u] = val[my];
        }
#pragma unroll
        for (int u = 0; u < CH; ++u) mu[u] = own(ix[u], mu[u]);
        fm_gather_slots<VEC, L, SQ, CH * L>(ix, mu, src, stride, kb, acc, sq);
    }
    for (; e < end; e += L) {
        const int64_t want = e + sub;
        const bool has = want < end;
        const int64_t my = has ? want : end - 1;
        int ix[1];
        float mu[1];
        ix[0] = idx[my];
        mu[0] = own(ix[0], has ? val[my] : 0.f);
        if constexpr (L <= 4) {
            fm_gather_slots<VEC, L, SQ, L>(ix, mu, src, stride, kb, acc, sq);
        } else {
            // wide groups: only the entries that exist, four gathers at a time
            const int nv = (int)((end - e) < L ? (end - e) : L);
            for (int t0 = 0; t0 < nv; t0 += 4) {
                float g[4][VEC];
                float mt[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int t = t0 + u < nv ? t0 + u : nv - 1;
                    const int it = __shfl(ix[0], t, L);
                    const float mm = __shfl(mu[0], t, L);
                    mt[u] = t0 + u < nv ? mm : 0.f;
                    fm_load_vec<VEC>(src + (int64_t)it * stride + kb, g[u]);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
#pragma unroll
                    for (int z = 0; z < VEC; ++z) {
                        acc[z] += mt[u] * g[u][z];
                        if constexpr (SQ) sq += (mt[u] * mt[u]) * (g[u][z] * g[u][z]);
                    }
                }
            }
        }
    }
}

// Column-side variant for packed aggregate rows [G_0..G_{K-1} | r | a | q | pad] whose [G | r] lies
// inside one 128-byte line: a group of L lanes, one lane wider than the latent values need, reads
// the row with a single request, and lane rl = K/VEC picks up r for the others.
// Per entry (row i, value x):
//   acc[z] += x r_i G_i[kb+z]     on the latent lanes,
//   gw += x r_i, s2 += x^2 r_i    on the scalar lane (the others keep 0).
template <int VEC, int L, bool NT, int S, int MAXB = 16, class IX, class XV>
__device__ __forceinline__ void fm_gather_slots_packed(const IX& ix, const XV& xv, const float* __restrict__ src,
                                                       int64_t stride, int kb, int rl, bool scalar_lane,
                                                       float (&acc)[VEC], float& gw, float& s2)
{
    constexpr int B = S < MAXB ? S : MAXB;
    fm_static_for<0, S / B>([&](auto bc) {
        constexpr int B0 = decltype(bc)::value * B;
        float g[B][VEC];
        float xt[B];
        fm_static_for<0, B>([&](auto sc) {
            constexpr int s = B0 + decltype(sc)::value;
            constexpr int u = s / L, T = s % L;
            const int it = fm_bcast_i<L, T>(ix[u]);
            xt[s - B0] = fm_bcast_f<L, T>(xv[u]);
            if constexpr (NT)
                fm_load_vec_nt<VEC>(src + (int64_t)it * stride + kb, g[s - B0]);
            else
                fm_load_vec<VEC>(src + (int64_t)it * stride + kb, g[s - B0]);
        });
#pragma unroll
        for (int s = 0; s < B; ++s) {
            const float r = __shfl(g[s][0], rl, L);
            const float m = xt[s] * r;
#pragma unroll
            for (int z = 0; z < VEC; ++z) acc[z] += m * g[s][z];
            if (scalar_lane) {
                gw += m;
                s2 += xt[s] * m;
            }
        }
    });
}

// kb: the caller clamps it so that lanes past the scalars re-read the row's last VEC floats
// (they discard their acc).
template <int VEC, int L, bool NT>
__device__ __forceinline__ void fm_col_accumulate_packed(const int32_t* __restrict__ idx, const float* __restrict__ val,
                                                         int64_t beg, int64_t end, const float* __restrict__ src,
                                                         int64_t stride, int sub, int kb, int rl, float (&acc)[VEC],
                                                         float& gw, float& s2)
{
    constexpr int CH = FmChunk<L>::CH;
    const bool scalar_lane = sub == rl;
    int64_t e = beg;
    for (; e + L * CH <= end; e += L * CH) {
        int ix[CH];
        float xv[CH];
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int64_t my = e + u * L + sub;
            ix[u] = idx[my];
            xv[u] = val[my];
        }
        fm_gather_slots_packed<VEC, L, NT, CH * L>(ix, xv, src, stride, kb, rl, scalar_lane, acc, gw, s2);
    }
    for (; e < end; e += L) {
        const int64_t want = e + sub;
        const bool has = want < end;
        const int64_t my = has ? want : end - 1;
        int ix[1];
        float xv[1];
        ix[0] = idx[my];
        xv[0] = has ? val[my] : 0.f;
        if constexpr (L <= 4) {
            fm_gather_slots_packed<VEC, L, NT, L>(ix, xv, src, stride, kb, rl, scalar_lane, acc, gw, s2);
        } else {
            // wide groups: only the entries that exist, four gathers at a time
            const int nv = (int)((end - e) < L ? (end - e) : L);
            for (int t0 = 0; t0 < nv; t0 += 4) {
                float g[4][VEC];
                float xt[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int t = t0 + u < nv ? t0 + u : nv - 1;
                    const int it = __shfl(ix[0], t, L);
                    const float x = __shfl(xv[0], t, L);
                    xt[u] = t0 + u < nv ? x : 0.f;
                    if constexpr (NT)
                        fm_load_vec_nt<VEC>(src + (int64_t)it * stride + kb, g[u]);
                    else
                        fm_load_vec<VEC>(src + (int64_t)it * stride + kb, g[u]);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float r = __shfl(g[u][0], rl, L);
                    const float m = xt[u] * r;
#pragma unroll
                    for (int z = 0; z < VEC; ++z) acc[z] += m * g[u][z];
                    if (scalar_lane) {
                        gw += m;
                        s2 += xt[u] * m;
                    }
                }
            }
        }
    }
}
