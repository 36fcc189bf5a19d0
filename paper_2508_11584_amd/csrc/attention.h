// Flash-style softmax attention for head_dim 64 on gfx950 (non-causal, all keys).
//
// Each wave owns 32 queries and walks the keys in tiles of 64.  The score tile is computed
// TRANSPOSED, S^T = K Q^T, so that in the 32x32 MFMA accumulator layout a lane holds 16 keys of
// ONE query (its column): the running max / sum of the online softmax are then in-lane
// reductions plus a single exchange between the two lane halves.  The probabilities stay in
// registers and feed the second product O^T = V^T P^T directly as its B operand; the A operand
// V^T comes from the transposed value buffer the QKV GEMM epilogue wrote (keys contiguous).
//
//   qk  [B*N][2*dim]  queries | keys, head h at columns 64h..64h+63 of each half
//   vt  [B*dim][npad] values transposed, npad = N rounded up to 64, padding columns zero
//   out [B*N][dim]
#pragma once
#include "common.h"
#include "gemm.h"

namespace vpe {

struct AttnArgs {
    const void* qk;
    const void* vt;
    void* out;
    int B, N, npad, dim, heads;
    float scale_log2e;   // (1 / sqrt(64)) * log2(e)
};

// --- per-type pieces: fragments for S^T = K Q^T and O^T = V^T P^T over a block of 32 keys
template <typename T> struct AttnMma;

template <> struct AttnMma<bf16> {
    static constexpr int QF = 4;                  // q fragments per lane (4 k-steps of 16 over dh = 64)
    typedef bf16x8 QFrag;
    static constexpr int ROWB = 128;              // bytes per 64-element row
    static __device__ __forceinline__ QFrag load_q(const bf16* qrow, int ks, int g) {
        return *reinterpret_cast<const QFrag*>(qrow + 16 * ks + 8 * g);
    }
    static __device__ __forceinline__ QFrag zero_q() { return QFrag{0, 0, 0, 0, 0, 0, 0, 0}; }
    // S^T block (32 keys x 32 queries) += K[keys][dh] Q^T
    static __device__ __forceinline__ void qk(f32x16& s, const char* sK, int krow, const QFrag* q, int g) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const bf16x8 a = *reinterpret_cast<const bf16x8*>(sK + (krow * 8 + swz(krow, 2 * ks + g)) * 16);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, q[ks], s, 0, 0, 0);
        }
    }
    // O^T block (32 dh x 32 queries) += V^T[dh][32 keys of block kb] P^T.  The k slot (g, kk) of
    // step s is key 16 s + 8 (kk / 4) + 4 g + kk % 4 -- exactly where accumulator element
    // v = 8 s + kk of the score block sits, so P needs no shuffle.
    static __device__ __forceinline__ void pv(f32x16& o, const char* sV, int drow, int kb, const f32x16& p, int g) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            bf16x8 b;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) b[kk] = (bf16)p[8 * s + kk];
            const int c0 = 4 * kb + 2 * s;     // 16-byte chunk holding keys 32 kb + 16 s .. + 7
            const bf16x4 lo = *reinterpret_cast<const bf16x4*>(sV + (drow * 8 + swz(drow, c0)) * 16 + 8 * g);
            const bf16x4 hi = *reinterpret_cast<const bf16x4*>(sV + (drow * 8 + swz(drow, c0 + 1)) * 16 + 8 * g);
            const bf16x8 a = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            o = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, o, 0, 0, 0);
        }
    }
};

template <> struct AttnMma<float> {
    static constexpr int QF = 4;                  // 4 macro steps of 16 dh
    struct QFrag { f32x4 lo, hi; };
    static constexpr int ROWB = 256;
    static __device__ __forceinline__ QFrag load_q(const float* qrow, int ks, int g) {
        QFrag f;
        f.lo = *reinterpret_cast<const f32x4*>(qrow + 16 * ks + 8 * g);
        f.hi = *reinterpret_cast<const f32x4*>(qrow + 16 * ks + 8 * g + 4);
        return f;
    }
    static __device__ __forceinline__ QFrag zero_q() { return QFrag{{0, 0, 0, 0}, {0, 0, 0, 0}}; }
    static __device__ __forceinline__ void qk(f32x16& s, const char* sK, int krow, const QFrag* q, int g) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const f32x4 lo = *reinterpret_cast<const f32x4*>(sK + (krow * 16 + swz(krow, 4 * ks + 2 * g)) * 16);
            const f32x4 hi = *reinterpret_cast<const f32x4*>(sK + (krow * 16 + swz(krow, 4 * ks + 2 * g + 1)) * 16);
#pragma unroll
            for (int i = 0; i < 4; ++i) s = __builtin_amdgcn_mfma_f32_32x32x2f32(lo[i], q[ks].lo[i], s, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < 4; ++i) s = __builtin_amdgcn_mfma_f32_32x32x2f32(hi[i], q[ks].hi[i], s, 0, 0, 0);
        }
    }
    // one MFMA per score element index v: k slot g is key 8 (v / 4) + 4 g + v % 4 of the block
    static __device__ __forceinline__ void pv(f32x16& o, const char* sV, int drow, int kb, const f32x16& p, int g) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            // keys 32 kb + 8 q4 + 4 g .. + 3  -> float chunk index (32 kb + 8 q4 + 4 g) / 4
            const int c = 8 * kb + 2 * q4 + g;
            const f32x4 a = *reinterpret_cast<const f32x4*>(sV + (drow * 16 + swz(drow, c)) * 16);
#pragma unroll
            for (int i = 0; i < 4; ++i) o = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], p[4 * q4 + i], o, 0, 0, 0);
        }
    }
};

template <typename T, int NW>
__global__ __launch_bounds__(64 * NW) void attention_kernel(const AttnArgs p) {
    constexpr int NT = 64 * NW;
    constexpr int CE = Elem<T>::CE;
    constexpr int CPR = 64 / CE;                 // 16-byte chunks per 64-element row
    constexpr int ROWB = AttnMma<T>::ROWB;
    constexpr int TILE = 64 * ROWB;
    constexpr int RPP = NT / CPR;                // rows loaded per pass
    constexpr int IT = 64 / RPP;
    static_assert(64 % RPP == 0, "loader pass must divide the tile");
    __shared__ __attribute__((aligned(16))) char smem[2 * TILE];
    char* sK = smem;
    char* sV = smem + TILE;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 5, li = lane & 31;
    const int bh = blockIdx.y, b = bh / p.heads, h = bh % p.heads;
    const int q0 = blockIdx.x * (32 * NW) + wave * 32;
    const int ld = 2 * p.dim;

    const T* __restrict__ qk = reinterpret_cast<const T*>(p.qk) + (int64_t)b * p.N * ld + h * 64;
    const T* __restrict__ kbase = qk + p.dim;
    const T* __restrict__ vt = reinterpret_cast<const T*>(p.vt) + ((int64_t)b * p.dim + h * 64) * p.npad;

    typename AttnMma<T>::QFrag q[4];
    {
        const int qi = q0 + li;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            q[ks] = qi < p.N ? AttnMma<T>::load_q(qk + (int64_t)qi * ld, ks, g) : AttnMma<T>::zero_q();
    }

    f32x16 o[2];
#pragma unroll
    for (int d = 0; d < 2; ++d)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[d][v] = 0.0f;
    float m_run = -INFINITY, l_run = 0.0f;

    const int lrow = tid / CPR, lchunk = tid % CPR;
    const int KT = p.npad / 64;
    u32x4 rk[IT], rv[IT];
    auto gload = [&](int kt) {
#pragma unroll
        for (int i = 0; i < IT; ++i) {
            const int r = lrow + i * RPP;
            const int key = kt * 64 + r;
            rk[i] = key < p.N ? ld_global_16(kbase + (int64_t)key * ld + lchunk * CE) : u32x4{0, 0, 0, 0};
            rv[i] = ld_global_16(vt + (int64_t)r * p.npad + kt * 64 + lchunk * CE);
        }
    };
    auto sstore = [&]() {
#pragma unroll
        for (int i = 0; i < IT; ++i) {
            const int r = lrow + i * RPP;
            const int phys = (lchunk & ~7) | swz(r, lchunk & 7);
            *reinterpret_cast<u32x4*>(sK + (r * CPR + phys) * 16) = rk[i];
            *reinterpret_cast<u32x4*>(sV + (r * CPR + phys) * 16) = rv[i];
        }
    };

    gload(0);
    for (int kt = 0; kt < KT; ++kt) {
        __syncthreads();           // everyone is done reading the previous tile
        sstore();
        __syncthreads();
        if (kt + 1 < KT) gload(kt + 1);

        f32x16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int v = 0; v < 16; ++v) s[kb][v] = 0.0f;
            AttnMma<T>::qk(s[kb], sK, kb * 32 + li, q, g);
        }
        if (kt == KT - 1) {        // keys past N only exist in the last tile
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = kt * 64 + kb * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                    if (key >= p.N) s[kb][v] = -INFINITY;
                }
        }
        float mx = s[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kb][v]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * p.scale_log2e);
        const float mc = m_new * p.scale_log2e;
        float psum = 0.0f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float e = __builtin_amdgcn_exp2f(fmaf(s[kb][v], p.scale_log2e, -mc));
                s[kb][v] = e;
                psum += e;
            }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int d = 0; d < 2; ++d)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[d][v] *= alpha;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int d = 0; d < 2; ++d) AttnMma<T>::pv(o[d], sV, d * 32 + li, kb, s[kb], g);
    }

    // each lane half summed its own keys; the query's denominator is the sum of both halves
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = 1.0f / l_tot;
    const int qi = q0 + li;
    if (qi < p.N) {
        T* orow = reinterpret_cast<T*>(p.out) + ((int64_t)b * p.N + qi) * p.dim + h * 64;
#pragma unroll
        for (int d = 0; d < 2; ++d)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                // O^T rows (dh) 32 d + 8 v4 + 4 g .. + 3 of this lane's query
                T* dst = orow + 32 * d + 8 * v4 + 4 * g;
#pragma unroll
                for (int i = 0; i < 4; ++i) dst[i] = from_f32<T>(o[d][4 * v4 + i] * inv);
            }
    }
}

template <typename T>
static inline hipError_t launch_attention_t(const AttnArgs& a, hipStream_t s) {
    // fewer waves per workgroup when there would otherwise be too few workgroups for 256 CUs
    const int bh = a.B * a.heads;
    if ((int64_t)cdiv(a.N, 128) * bh >= 512) {
        hipLaunchKernelGGL((attention_kernel<T, 4>), dim3(cdiv(a.N, 128), bh), dim3(256), 0, s, a);
    } else if ((int64_t)cdiv(a.N, 64) * bh >= 256) {
        hipLaunchKernelGGL((attention_kernel<T, 2>), dim3(cdiv(a.N, 64), bh), dim3(128), 0, s, a);
    } else {
        hipLaunchKernelGGL((attention_kernel<T, 1>), dim3(cdiv(a.N, 32), bh), dim3(64), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace vpe
