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

// The loader prefetches one iteration (KW key tiles) ahead without clamping, so a workgroup with KW key waves
// reads up to 2 KW 64 key rows past the last token of qk and as many elements past the end of vt (tiles that do
// not exist); both buffers must be readable that far.  What is read there is never used.  `pad` states how many
// rows of qk / elements of vt past their ends the caller made readable; a launch whose shape needs more is refused.
constexpr int ATTN_MAX_KW = 4;                        // widest key split of any instantiation
constexpr int ATTN_PAD = 2 * ATTN_MAX_KW * 64;        // rows / elements a caller has to provide for any shape
struct AttnArgs {
    const void* qk;
    const void* vt;
    void* out;
    int B, N, npad, dim, heads;
    float scale_log2e;   // (1 / sqrt(64)) * log2(e)
    int pad;             // readable rows of qk / elements of vt past their ends
    int shared_gpu;      // the launch runs beside other streams' kernels (several encoder lanes): prefer a shape that
                         // leaves room on its CUs over the fastest one on an empty GPU
};

// Exchange between the two halves of a wave without going through LDS (v_permlane32_swap): both operands are the
// lane's own value, after the swap one holds the lower half's values in all 64 lanes and the other the upper half's.
__device__ __forceinline__ float halves_max(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float halves_sum(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

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
    // Both 32-key blocks of a tile at once: S0^T, S1^T = K[0..31], K[32..63] times Q^T.  The two accumulation chains
    // alternate (consecutive MFMAs are independent) and the K fragments of k-step ks + 1 are read while the MFMAs of
    // step ks run, instead of read - wait - multiply eight times in a row.
    static __device__ __forceinline__ void qk2(f32x16& s0, f32x16& s1, const char* sK, int li, const QFrag* q, int g) {
        // Accumulator row r of the score block is fed from key row pi(r) = r with bits 2 and 3 exchanged: lane half g
        // then holds, for k-step s of the second product, the eight CONSECUTIVE keys 16 s + 8 g .. + 7 (see pv_tile)
        const int kr = (li & 0x13) | ((li & 8) >> 1) | ((li & 4) << 1);
        const int sw = (kr >> 1) & 7;                      // rows kr and kr + 32 share the swizzle term
        const char* r0 = sK + kr * 128;
        const char* r1 = r0 + 32 * 128;
        bf16x8 a[2][2];
        a[0][0] = *reinterpret_cast<const bf16x8*>(r0 + ((g ^ sw) * 16));
        a[0][1] = *reinterpret_cast<const bf16x8*>(r1 + ((g ^ sw) * 16));
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks < 3) {
                a[(ks + 1) & 1][0] = *reinterpret_cast<const bf16x8*>(r0 + (((2 * ks + 2 + g) ^ sw) * 16));
                a[(ks + 1) & 1][1] = *reinterpret_cast<const bf16x8*>(r1 + (((2 * ks + 2 + g) ^ sw) * 16));
            }
            __builtin_amdgcn_sched_barrier(0);         // the reads above stay ahead of the MFMAs below
            s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks & 1][0], q[ks], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks & 1][1], q[ks], s1, 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // Key (within its 32-key block) of accumulator element v of the score block in lane half g, under the row
    // permutation of qk2.
    static __device__ __forceinline__ int key_of(int v, int g) { return 16 * (v >> 3) + 8 * g + (v & 7); }
    // O^T (64 dh x 32 queries, two accumulators) += V^T[dh][64 keys] P^T, and the row sums of P.  Four k-steps of 16
    // keys; the k slot (g, kk) of step (kb, s) is key 32 kb + 16 s + 8 g + kk -- where accumulator element
    // v = 8 s + kk of score block kb sits, so P needs no shuffle, and a lane's eight keys are one 16-byte chunk of
    // a V^T row (one conflict-free ds_read_b128 per accumulator and step).  The reads of step + 1 are issued before
    // the MFMAs of step.
    // Row sums on the matrix pipe (LM): ones[32 x 16] P^T adds the 16 keys of a k-step for every query, in every
    // row of the accumulator (lane halves included), using the same rounded probabilities as the numerator; four
    // of these per tile replace 32 VALU additions per lane.
    static constexpr bool MFMA_ROWSUM = true;
    // `sc` holds the raw scores; element e becomes 2^(sc[e] * scale - ref).  The exponentials of step + 1 are issued
    // behind the MFMAs of step, so the vector pipe works on them while the matrix pipe runs.  psum (LM == false)
    // receives the lane's sum of probabilities.
    template <bool LM>
    static __device__ __forceinline__ void pv_tile(f32x16& o0, f32x16& o1, f32x16& l, float& psum, const char* sV, int li,
                                                   f32x16* sc, float scale, float ref, int g) {
        const bf16x8 ones = {(bf16)1.0f, (bf16)1.0f, (bf16)1.0f, (bf16)1.0f, (bf16)1.0f, (bf16)1.0f, (bf16)1.0f, (bf16)1.0f};
        const int sw = (li >> 1) & 7;                      // rows li and li + 32 share the swizzle term
        const char* r0 = sV + li * 128;
        const char* r1 = r0 + 32 * 128;
        auto probs = [&](int st) {
            bf16x8 b;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                const float e = __builtin_amdgcn_exp2f(fmaf(sc[st >> 1][8 * (st & 1) + kk], scale, -ref));
                if (!LM) psum += e;
                b[kk] = (bf16)e;
            }
            return b;
        };
        bf16x8 a[2][2], b[2];
        a[0][0] = *reinterpret_cast<const bf16x8*>(r0 + ((g ^ sw) * 16));
        a[0][1] = *reinterpret_cast<const bf16x8*>(r1 + ((g ^ sw) * 16));
        b[0] = probs(0);
#pragma unroll
        for (int st = 0; st < 4; ++st) {
            if (st < 3) {
                a[(st + 1) & 1][0] = *reinterpret_cast<const bf16x8*>(r0 + (((2 * st + 2 + g) ^ sw) * 16));
                a[(st + 1) & 1][1] = *reinterpret_cast<const bf16x8*>(r1 + (((2 * st + 2 + g) ^ sw) * 16));
            }
            __builtin_amdgcn_sched_barrier(0);
            o0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[st & 1][0], b[st & 1], o0, 0, 0, 0);
            o1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[st & 1][1], b[st & 1], o1, 0, 0, 0);
            if (LM) l = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, b[st & 1], l, 0, 0, 0);
            if (st < 3) b[(st + 1) & 1] = probs(st + 1);
            // one MFMA, then a third of the next step's exponentials and conversions, three times
#pragma unroll
            for (int i = 0; i < 3; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x402, 8, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
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
    static __device__ __forceinline__ void qk2(f32x16& s0, f32x16& s1, const char* sK, int li, const QFrag* q, int g) {
        qk(s0, sK, li, q, g);
        qk(s1, sK, 32 + li, q, g);
    }
    static __device__ __forceinline__ int key_of(int v, int g) { return 8 * (v >> 2) + 4 * g + (v & 3); }
    template <bool LM>
    static __device__ __forceinline__ void pv_tile(f32x16& o0, f32x16& o1, f32x16&, float& psum, const char* sV, int li,
                                                   f32x16* sc, float scale, float ref, int g) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                sc[kb][v] = __builtin_amdgcn_exp2f(fmaf(sc[kb][v], scale, -ref));
                psum += sc[kb][v];
            }
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            pv(o0, sV, li, kb, sc[kb], g);
            pv(o1, sV, 32 + li, kb, sc[kb], g);
        }
    }
    // one MFMA per score element index v: k slot g is key 8 (v / 4) + 4 g + v % 4 of the block
    static constexpr bool MFMA_ROWSUM = false;
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

// Workgroup shape: QW x KW waves.  Wave (qw, kw) owns QB blocks of 32 queries (query group qw) and
// the key tiles t with t % KW == kw.  Each iteration stages KW key tiles and KW value tiles in LDS,
// loaded by all threads; waves of the same kw share their tile across query groups.  At the end
// the KW partial results of a query group are merged in LDS by its kw = 0 wave (fixed order, so
// results are deterministic).  KW > 1 gives small problems enough waves to fill 1024 SIMDs;
// QW > 1 and QB = 2 cut the L2 -> LDS traffic per query on large ones.
// Launch bound: at least two waves per SIMD wherever the kernel fits 256 registers.  Besides the occupancy, this
// is what makes the compiler keep the MFMA accumulators in ordinary vector registers: with up to 512 registers
// allowed it places them in the accumulation-register file, and since the softmax works on the scores with
// vector instructions every tile then pays ~190 register-file moves per lane (measured on the four-wave shapes:
// 158 + 48 registers and 300 vector instructions per tile without the bound, 164 + 0 and 105 with it).  Two
// shapes would spill under the bound and keep the old one.
template <typename T, int KW>
constexpr bool attn_double_buffered() { return 2 * KW * 2 * 64 * AttnMma<T>::ROWB <= 128 * 1024; }

template <typename T, int QB, int QW, int KW>
constexpr int attn_min_waves() { return (QW * KW == 4 && (QB == 2 || (sizeof(T) == 4 && KW == 4))) ? 1 : 2; }

template <typename T, int QB, int QW, int KW>
__global__ __launch_bounds__(64 * QW * KW, (attn_min_waves<T, QB, QW, KW>())) void attention_kernel(const AttnArgs p) {
    constexpr int NW = QW * KW, NT = 64 * NW;
    static_assert(KW <= ATTN_MAX_KW, "the loader's overshoot is budgeted for at most ATTN_MAX_KW key waves");
    constexpr int CE = Elem<T>::CE;
    constexpr int CPR = 64 / CE;                 // 16-byte chunks per 64-element row
    constexpr int ROWB = AttnMma<T>::ROWB;
    constexpr int TILE = 64 * ROWB;
    constexpr int CH = KW * 2 * 64 * CPR / NT;   // chunks per thread per iteration
    constexpr int STAGE = KW * 2 * TILE;         // K and V tiles of one iteration
    constexpr bool DB = attn_double_buffered<T, KW>();
    static_assert((KW * 2 * 64 * CPR) % NT == 0 && NT % CPR == 0, "loader mapping");
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int qw = wave % QW, kw = wave / QW;
    const int g = lane >> 5, li = lane & 31;
    // One-dimensional grid, (image, head)-major: the hardware deals consecutive workgroups round-robin to the 8 XCDs,
    // so ids are remapped to give each XCD one contiguous range -- all query blocks of an (image, head) pair then run
    // on the same XCD and its keys and values are fetched into that L2 once, not into all eight (measured at ViT-g x8:
    // 615 MB fetched per launch against 135 MB of operands before the remapping).
    const int nqb = cdiv(p.N, 32 * QB * QW);
    const int lin = xcd_contiguous(blockIdx.x, gridDim.x);
    const int bh = lin / nqb, b = bh / p.heads, h = bh % p.heads;
    const int q0 = (lin % nqb) * (32 * QB * QW) + qw * 32 * QB;
    const int ld = 2 * p.dim;

    const T* __restrict__ qk = reinterpret_cast<const T*>(p.qk) + (int64_t)b * p.N * ld + h * 64;
    const T* __restrict__ kbase = qk + p.dim;
    const T* __restrict__ vt = reinterpret_cast<const T*>(p.vt) + ((int64_t)b * p.dim + h * 64) * p.npad;

    typename AttnMma<T>::QFrag q[QB][4];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int qi = q0 + qb * 32 + li;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
            q[qb][ks] = qi < p.N ? AttnMma<T>::load_q(qk + (int64_t)qi * ld, ks, g) : AttnMma<T>::zero_q();
    }

    // denominators: on the matrix pipe where the type and the register budget allow it (complete sums, every
    // accumulator row the same), else per lane half in l_run
    constexpr bool LMFMA = AttnMma<T>::MFMA_ROWSUM && QB == 1;
    f32x16 lacc[LMFMA ? QB : 1];
    f32x16 o[QB][2];
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.0f;
        if (LMFMA) {
#pragma unroll
            for (int v = 0; v < 16; ++v) lacc[qb][v] = 0.0f;
        }
#pragma unroll
        for (int d = 0; d < 2; ++d)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[qb][d][v] = 0.0f;
    }

    const int KT = p.npad / 64;
    const int NIT = (KT + KW - 1) / KW;
    const int lchunk = tid % CPR;
    u32x4 rg[DB ? 1 : CH];                             // register staging: single-buffer shapes only
    // chunk i of this thread: linear index tid + i NT over (tile j, K|V, row, chunk).  Its address advances by a
    // fixed step per iteration (KW tiles), so the loader keeps one running pointer per chunk instead of
    // recomputing tile, row and clamps each time.  Nothing is clamped: tiles past the last one and key rows past
    // N are read from whatever follows (the next image's keys, the buffers' padding -- see AttnArgs) and never
    // used: scores of keys >= N are overwritten with -inf, waves skip tiles >= KT.
    // Thread part of the address (its row within a pass and its chunk) in two pointers; tile, K|V and pass of
    // chunk i are compile-time constants, the advance per iteration is wave-uniform: scalar arithmetic only.
    constexpr int RPP = NT / CPR;                      // rows per loader pass
    static_assert(64 % RPP == 0, "a pass must not straddle tiles");
    const T* kthr = kbase + (int64_t)(tid / CPR) * ld + lchunk * CE;
    const T* vthr = vt + (int64_t)(tid / CPR) * p.npad + lchunk * CE;
    int64_t kadv = 0, vadv = 0;
    auto gload = [&]() {                               // loads the next iteration's tiles
#pragma unroll
        for (int i = 0; i < (DB ? 0 : CH); ++i) {
            const int r0 = (i * RPP) & 63, which = ((i * RPP) >> 6) & 1, j = (i * RPP) >> 7;
            const T* src = which ? vthr + (int64_t)r0 * p.npad + j * 64 + vadv
                                 : kthr + (int64_t)(j * 64 + r0) * ld + kadv;
            rg[i] = ld_global_16(src);
        }
        kadv += (int64_t)KW * 64 * ld;
        vadv += KW * 64;
    };
    auto sstore = [&](char* base) {
#pragma unroll
        for (int i = 0; i < (DB ? 0 : CH); ++i) {
            const int idx = (tid + i * NT) / CPR;
            const int row = idx & 63;
            const int phys = (lchunk & ~7) | swz(row, lchunk & 7);
            *reinterpret_cast<u32x4*>(base + (idx >> 6) * TILE + (row * CPR + phys) * 16) = rg[i];
        }
    };

    // Double-buffered shapes load straight into LDS (global_load_lds_dwordx4: no staging registers, no ds_write).
    // One instruction of a wave fills 1 KB = RPI consecutive rows of a tile; lane l lands on row l / CPR, physical
    // chunk l % CPR of that row group, so it fetches the logical chunk that belongs there under the swizzle.
    // Instruction i of wave w fills slot w + NW i of the stage (tile i / PPT, pass i % PPT over its row groups):
    // a lane's row within the tile is (w + NW pass) RPI + l / CPR -- the passes differ by multiples of 16 rows, which
    // leave the swizzle term unchanged, so one logical chunk and two thread pointers serve every instruction.
    constexpr int RPI = 1024 / ROWB, G = TILE / 1024;  // rows per instruction, instructions per tile
    constexpr int PPT = G / NW > 0 ? G / NW : 1;       // passes of the workgroup over one tile
    constexpr int NDMA = KW * 2 * G / NW;              // instructions per wave per iteration
    static_assert(!DB || (G % NW == 0 && (NW * RPI) % 16 == 0) || NW == G, "loader mapping of the direct-to-LDS path");
    const int drow = wave * RPI + lane / CPR;
    const int dlc = ((lane % CPR) & ~7) | (((lane % CPR) & 7) ^ ((drow >> 1) & 7));
    const T* kdma = kbase + (int64_t)drow * ld + dlc * CE;
    const T* vdma = vt + (int64_t)drow * p.npad + dlc * CE;
    auto dma = [&](char* base, int it) {               // tiles of iteration `it` into the stage at `base`
        const int64_t ka = (int64_t)it * KW * 64 * ld;
        const int va = it * KW * 64;
#pragma unroll
        for (int i = 0; i < (DB ? NDMA : 0); ++i) {
            const int ti = i / PPT, pass = i % PPT, j = ti >> 1, which = ti & 1, r0 = pass * NW * RPI;
            const T* src = which ? vdma + (int64_t)r0 * p.npad + j * 64 + va : kdma + (int64_t)(j * 64 + r0) * ld + ka;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)(base + (wave + NW * i) * 1024), 16, 0, 0);
        }
    };
    // Two buffers: the loads of iteration it + 1 are issued at the top of iteration it into the buffer that was read
    // in iteration it - 1, and one barrier per iteration is enough (everyone has finished reading buffer b, and the
    // loads into buffer b ^ 1 have landed).  Shapes whose two buffers would not fit the CU's LDS keep one buffer,
    // register staging and two barriers.
    if constexpr (DB) {
        dma(smem, 0);
        __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): the loads into LDS have landed
        __syncthreads();
    } else {
        gload();
    }
    for (int it = 0; it < NIT; ++it) {
        const char* stage = smem;
        if constexpr (DB) {
            if (it + 1 < NIT) dma(smem + ((it + 1) & 1) * STAGE, it + 1);
            stage = smem + (it & 1) * STAGE;
        } else {
            __syncthreads();           // everyone is done reading the previous tiles
            sstore(smem);
            __syncthreads();
            if (it + 1 < NIT) gload();
        }
        const int t = it * KW + kw;
        if (t < KT) {                  // (a wave without a tile in the last iteration still takes part in the barriers)
            const char* sK = stage + (kw * 2) * TILE;
            const char* sV = sK + TILE;
            const bool last = t == KT - 1;     // keys past N only exist in the last tile
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                f32x16 s[2];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) s[kb][v] = 0.0f;
                AttnMma<T>::qk2(s[0], s[1], sK, li, q[qb], g);
                if (last) {
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int key = t * 64 + kb * 32 + AttnMma<T>::key_of(v, g);
                            if (key >= p.N) s[kb][v] = -INFINITY;
                        }
                }
                float mx = s[0][0];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kb][v]);
                mx = halves_max(mx);
                // Lazy rescaling: m_run is the reference the exponentials are taken against (in log2 units), not
                // necessarily the running maximum.  It only moves when a query's maximum has grown by more than 8
                // (probabilities stay <= 2^8, exact in fp32 and harmless in bf16), which after the first tile is
                // rare -- and then the whole wave skips the 32 multiplications of the accumulator.  On the first
                // tile the reference is -inf, alpha = 0 and the (zero) accumulators are overwritten.
                const float mxs = mx * p.scale_log2e;
                const bool grow = mxs > m_run[qb] + 8.0f;
                if (__any(grow)) {
                    const float m_new = grow ? mxs : m_run[qb];
                    const float alpha = __builtin_amdgcn_exp2f(m_run[qb] - m_new);
                    l_run[qb] *= alpha;
                    m_run[qb] = m_new;
                    if (LMFMA) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) lacc[qb][v] *= alpha;
                    }
#pragma unroll
                    for (int d = 0; d < 2; ++d)
#pragma unroll
                        for (int v = 0; v < 16; ++v) o[qb][d][v] *= alpha;
                }
                float psum = 0.0f;
                AttnMma<T>::template pv_tile<LMFMA>(o[qb][0], o[qb][1], lacc[LMFMA ? qb : 0], psum, sV, li, s, p.scale_log2e, m_run[qb], g);
                if (!LMFMA) l_run[qb] += psum;
            }
        }
        if constexpr (DB) {
            __builtin_amdgcn_s_waitcnt(0x0F70);
            __syncthreads();
        }
    }

    if (LMFMA) {
        // the matrix-pipe sums are complete in both lane halves; the code below adds the halves, so each takes half
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) l_run[qb] = 0.5f * lacc[qb][0];
    }

    if constexpr (KW > 1) {
        // merge the KW partial (max, sum, O) triples of each query group, lane by lane
        constexpr int PER = QB * (32 + 2) * 64;          // floats per wave: O (32 per lane), m, l
        float* red = reinterpret_cast<float*>(smem);
        __syncthreads();
        if (kw > 0) {
            float* dst = red + ((kw - 1) * QW + qw) * PER + lane;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
                for (int d = 0; d < 2; ++d)
#pragma unroll
                    for (int v = 0; v < 16; ++v) dst[(qb * 34 + d * 16 + v) * 64] = o[qb][d][v];
                dst[(qb * 34 + 32) * 64] = m_run[qb];
                dst[(qb * 34 + 33) * 64] = l_run[qb];
            }
        }
        __syncthreads();
        if (kw > 0) return;
        for (int k = 1; k < KW; ++k) {
            const float* src = red + ((k - 1) * QW + qw) * PER + lane;
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                const float mk = src[(qb * 34 + 32) * 64], lk = src[(qb * 34 + 33) * 64];
                const float m_new = fmaxf(m_run[qb], mk);
                const float a = __builtin_amdgcn_exp2f(m_run[qb] - m_new);      // references are in log2 units
                const float bsc = __builtin_amdgcn_exp2f(mk - m_new);
#pragma unroll
                for (int d = 0; d < 2; ++d)
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        o[qb][d][v] = o[qb][d][v] * a + src[(qb * 34 + d * 16 + v) * 64] * bsc;
                l_run[qb] = l_run[qb] * a + lk * bsc;
                m_run[qb] = m_new;
            }
        }
    }

    // each lane half summed its own keys; the query's denominator is the sum of both halves
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float l_tot = halves_sum(l_run[qb]);
        const float inv = 1.0f / l_tot;
        const int qi = q0 + qb * 32 + li;
        if (qi < p.N) {
            T* orow = reinterpret_cast<T*>(p.out) + ((int64_t)b * p.N + qi) * p.dim + h * 64;
#pragma unroll
            for (int d = 0; d < 2; ++d)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    // O^T rows (dh) 32 d + 8 v4 + 4 g .. + 3 of this lane's query
                    T* dst = orow + 32 * d + 8 * v4 + 4 * g;
#pragma unroll
                    for (int i = 0; i < 4; ++i) dst[i] = from_f32<T>(o[qb][d][4 * v4 + i] * inv);
                }
        }
    }
}

template <typename T, int QB, int QW, int KW>
static inline hipError_t launch_attention_variant(const AttnArgs& a, hipStream_t s, bool configure_only) {
    constexpr int TILE = 64 * AttnMma<T>::ROWB;
    constexpr int kv = (attn_double_buffered<T, KW>() ? 2 : 1) * KW * 2 * TILE, red = (KW - 1) * QW * QB * 34 * 64 * 4;
    constexpr int lds = kv > red ? kv : red;
    static bool configured = false;       // opt in to more than 64 KB of LDS once per instantiation
    if (!configured) {
        hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&attention_kernel<T, QB, QW, KW>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (rc != hipSuccess) return rc;
        configured = true;
    }
    if (configure_only) return hipSuccess;
    if (a.pad < 2 * KW * 64 || a.npad % 64 || a.npad < a.N || a.dim != a.heads * 64) return hipErrorInvalidValue;
    hipLaunchKernelGGL((attention_kernel<T, QB, QW, KW>), dim3(cdiv(a.N, 32 * QB * QW) * a.B * a.heads),
                       dim3(64 * QW * KW), lds, s, a);
    return hipGetLastError();
}

}  // namespace vpe
