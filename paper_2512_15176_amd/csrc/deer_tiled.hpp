// LDS-tiled GEMM for passes with many rows (prefill chunks, wide batches): out = X W with the same operands,
// layouts and fused epilogues as the weight-streaming GEMM, but blocked for the matrix cores instead of for
// HBM: a workgroup owns 256 rows x 256 columns, both operands travel HBM/L2 -> LDS once per workgroup with
// direct-to-LDS loads (fragments are stored in MFMA register order in memory, so a fragment is a plain 1 KB
// copy), and every wave multiplies a 64 x 128 sub-tile out of LDS.
//
// Per k-step of 16 a workgroup moves 24 KB (8 weight fragments, 8 row tiles x (hi, lo)) for 128 MFMAs, against
// 64 KB for the same work in the streaming kernel, which re-reads the weights per 64 rows.
#pragma once
#include "deer_kernels.hpp"

namespace deer {

constexpr int TG_RT = 8;        // row tiles per workgroup (256 rows): wave (w >> 1) owns two of them
#ifndef DEER_TG_KST
#define DEER_TG_KST 2
#define DEER_TG_NST 3
#endif
constexpr int TG_KST = DEER_TG_KST;   // k-steps per stage
constexpr int TG_NST = DEER_TG_NST;   // stage buffers: all but one are on their way while one is multiplied
static_assert(TG_NST >= 3 && TG_NST <= 6 && TG_KST * TG_NST <= 6, "stage buffers must fit LDS");
constexpr int TG_FRAGS = 24;    // fragments per k-step: 8 weight column tiles, 8 row tiles hi, 8 row tiles lo
constexpr int TG_LPW = TG_KST * TG_FRAGS / 8;   // direct-to-LDS loads per wave and stage

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // a register quad as the inline assembly sees it
// LDS byte address of a __shared__ object
__device__ __forceinline__ uint32_t lds_addr(const void *p) {
    return (uint32_t)(size_t)(const void __attribute__((address_space(3))) *)p;
}
template <int OFF>
__device__ __forceinline__ void lds_read16(u32x4 &v, uint32_t addr) {
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
}
// one k-step's fragments of a wave: 4 weight column tiles, 2 row tiles (hi, lo)
struct TiledFrags { u32x4 wf[4], xh[2], xl[2]; };
// byte offsets inside a stage: fragment f of k-step kst at (kst * 24 + f) KB; sbw points at this wave's first weight
// fragment, sbx at its first hi fragment (the lo fragments lie 8 KB further)
template <int KOFF>
__device__ __forceinline__ void tiled_read_frags(TiledFrags &f, uint32_t sbw, uint32_t sbx) {
    lds_read16<KOFF + 0>(f.wf[0], sbw); lds_read16<KOFF + 1024>(f.wf[1], sbw);
    lds_read16<KOFF + 2048>(f.wf[2], sbw); lds_read16<KOFF + 3072>(f.wf[3], sbw);
    lds_read16<KOFF + 0>(f.xh[0], sbx); lds_read16<KOFF + 1024>(f.xh[1], sbx);
    lds_read16<KOFF + 8192>(f.xl[0], sbx); lds_read16<KOFF + 9216>(f.xl[1], sbx);
}
// the fragments are valid after this point (they pass through the wait as operands, so no use can move above it)
__device__ __forceinline__ void lds_wait8(TiledFrags &f) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f.wf[0]), "+v"(f.wf[1]), "+v"(f.wf[2]), "+v"(f.wf[3]), "+v"(f.xh[0]), "+v"(f.xh[1]), "+v"(f.xl[0]), "+v"(f.xl[1]));
}

struct TiledSmem {
    union {
        uint4 st[TG_NST][TG_KST * TG_FRAGS * 64];                       // 3 x 48 KB
        struct { float tile[32 * RED_STRIDE]; float scratch[256]; } ep;   // epilogue staging, after the K loop
    };
    float rstd[TG_RT * 32];
};

// The workgroups that run on one XCD at the same time form a patch of 4 row blocks x 8 column pairs, so that
// per k-step the XCD's L2 fetches 4 activation slabs and 8 weight slabs and serves them 8 and 4 times.
// Workgroup ids 8 apart share an XCD: id = 8 * (32 * patch_in_xcd + i) + xcd, i = 4 * column + row inside the patch.
struct TiledMap { int rb, cp; bool valid; };
__device__ __forceinline__ TiledMap tiled_map(int lin, int nrb, int ncp) {
    const int x = lin & 7, q = lin >> 3;
    const int P = (q >> 5) * 8 + x, i = q & 31;
    const int prow = (nrb + 3) >> 2;   // patches along the rows
    const int pr = P % opaque_s(prow), pc = P / opaque_s(prow);
    TiledMap m;
    m.rb = pr * 4 + (i & 3);
    m.cp = pc * 8 + (i >> 2);
    m.valid = m.rb < nrb && m.cp < ncp;
    return m;
}

// ncg: 128-column groups of the matrix; nrt: row tiles of the pass (tile index ct = 0 .. nrt - 1 maps to the
// pass tile a.mt0 + ct * a.mt_stride).  Grid: 1-D, tiled_blocks(nrt, ncg) workgroups of 512 threads.  a.S is 1.
template <int EPI>
__global__ __launch_bounds__(512) void k_gemm_tiled(const GemmArgs a, int ncg, int nrt) {
    __shared__ __attribute__((aligned(16))) TiledSmem sm;
    const int tidx = opaque_tid();
    const int w = __builtin_amdgcn_readfirstlane(tidx >> 6), lane = tidx & 63;
    const int wr = w >> 1, wc = w & 1;
    const int nrb = (nrt + TG_RT - 1) / TG_RT, ncp = (ncg + 1) >> 1;
    const TiledMap mp = tiled_map(blockIdx.x, nrb, ncp);
    if (!mp.valid) return;
    const int KS = a.KS, nst = KS / TG_KST;
    const int ct_last = a.N / 32 - 1;

    // Requests this wave's share of stage `it` (fragments f = 6 w .. 6 w + 5 of the 48).  Column and row tiles
    // past the matrix repeat the last valid one (their products are not used).
    auto stage = [&](int buf, int it) {
        int lo16 = lane;   // lane offset inside a fragment, rebuilt here (not kept live across the K loop)
        asm volatile("" : "+v"(lo16));
#pragma unroll
        for (int i = 0; i < TG_LPW; ++i) {
            const int f = w * TG_LPW + i, kst = f / TG_FRAGS, fr = f % TG_FRAGS;
            const int ks = it * TG_KST + kst;
            const uint4 *src;
            if (fr < 8) {
                const int ctile = min(mp.cp * 8 + fr, ct_last);
                src = a.W + ((size_t)ctile * KS + ks) * 64 + lo16;
            } else {
                const int rt = min(mp.rb * TG_RT + ((fr - 8) & 7), nrt - 1);
                const size_t tl = (size_t)(a.mt0 + rt * a.mt_stride);
                src = (fr < 16 ? a.Xhi : a.Xlo) + (tl * KS + ks) * 64 + lo16;
            }
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)src,
                                             (void __attribute__((address_space(3))) *)(sm.st[buf] + (kst * TG_FRAGS + fr) * 64), 16, 0, 0);
        }
    };

    f32x16 acc[2][4];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nb][r] = 0.f;

    static_assert(TG_KST == 2 && TG_NST == 3, "the loop below is written for two k-steps per stage and three buffers");
#pragma unroll
    for (int i = 0; i < TG_NST; ++i)
        if (i < nst) stage(i, i);
    // RMSNorm factors of the workgroup's rows (their sums of squares were finished by the previous kernel)
    if (EPI != EPI_RESID) {
#pragma unroll 1
        for (int rt = 0; rt < TG_RT; ++rt) {
            const int ct = min(mp.rb * TG_RT + rt, nrt - 1);
            tile_rstd<false>(a.ssq_in, sm.rstd + 32 * rt, (a.mt0 + ct * a.mt_stride) * 32, a.ncg_in, a.d_in, a.eps);
        }
    }

    // The fragments are read with LDS instructions the compiler does not see as such: before a read of memory
    // that direct-to-LDS loads may write it waits for ALL loads in flight (vmcnt(0)), the stages requested
    // ahead included, and the ring would never be more than one stage deep.  The counted waits and the
    // barriers below are what orders these reads after the loads of their own stage.
    // Schedule of stage `it` (steady state; two stages are on their way all the time):
    //   read k-step 1 | multiply k-step 0 | wait: stage it+1 has landed | barrier: everybody has read stage it |
    //   request stage it+3 into the buffer of stage it | read k-step 0 of stage it+1 | multiply k-step 1
    // so the LDS reads of a k-step always run under the products of the one before, also across the barrier.
    const uint32_t lane16 = lane * 16, wofs = wc * 4096, xofs = 8192 + wr * 2048;
    auto mul16 = [&](const TiledFrags &f) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                acc[mt][nb] = mfma32(__builtin_bit_cast(uint4, f.xh[mt]), __builtin_bit_cast(uint4, f.wf[nb]), acc[mt][nb]);
                acc[mt][nb] = mfma32(__builtin_bit_cast(uint4, f.xl[mt]), __builtin_bit_cast(uint4, f.wf[nb]), acc[mt][nb]);
            }
    };
    TiledFrags fa, fb;
    if (nst > 2) wait_loads<2 * TG_LPW>(); else if (nst > 1) wait_loads<TG_LPW>(); else wait_loads<0>();
    barrier_keep_loads();   // stage 0 is in LDS
    {
        const uint32_t sb = lds_addr(sm.st[0]) + lane16;
        tiled_read_frags<0>(fa, sb + wofs, sb + xofs);
        lds_wait8(fa);
    }
    for (int it = 0; it < nst; ++it) {
        const uint32_t sb = lds_addr(sm.st[it % TG_NST]) + lane16;
        tiled_read_frags<TG_FRAGS * 1024>(fb, sb + wofs, sb + xofs);
        mul16(fa);
        __builtin_amdgcn_sched_barrier(0);   // the products are queued before the wave waits for its next fragments
        lds_wait8(fb);
        const bool more = it + 1 < nst;
        if (more) {
            if (it + 2 < nst) wait_loads<TG_LPW>(); else wait_loads<0>();   // stage it+1 has landed (it+2 may be on its way)
            barrier_keep_loads();   // everybody's share of stage it+1 is in LDS, and everybody has read stage it
            if (it + TG_NST < nst) stage(it % TG_NST, it + TG_NST);
            const uint32_t sn = lds_addr(sm.st[(it + 1) % TG_NST]) + lane16;
            tiled_read_frags<0>(fa, sn + wofs, sn + xofs);
        }
        mul16(fb);
        __builtin_amdgcn_sched_barrier(0);
        if (more) lds_wait8(fa);
    }
    __syncthreads();   // the stage buffers have been read: the epilogue staging below reuses them

    // 16 (row tile, column group) results, one at a time through the row-major staging tile and the same
    // epilogues as the streaming kernel
    const int half = lane >> 5, cl = lane & 31;
    float hreg[8];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
#pragma unroll 1
        for (int o = 0; o < 8; ++o) {
            const int rt = (o >> 1) * 2 + mt, cgi = o & 1;
            const int ct = mp.rb * TG_RT + rt, cg = mp.cp * 2 + cgi;
            if (ct >= nrt || cg >= ncg) continue;   // uniform over the workgroup
            if (EPI == EPI_RESID) resid_prefetch<false>(a, hreg, cg, a.mt0 + ct * a.mt_stride);
            if (w == o) {
#pragma unroll
                for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        sm.ep.tile[mfma_row(r, half) * RED_STRIDE + nb * 32 + cl] = acc[mt][nb][r];
            }
            __syncthreads();
            run_epilogue<EPI, false, true>(a, sm.ep.tile, sm.rstd + 32 * rt, sm.ep.scratch, hreg, cg, ct);
            __syncthreads();
        }
    }
}

inline int tiled_blocks(int nrt, int ncg) {
    const int nrb = (nrt + TG_RT - 1) / TG_RT, ncp = (ncg + 1) / 2;
    const int patches = ((nrb + 3) / 4) * ((ncp + 7) / 8);
    return ((patches + 7) / 8) * 8 * 32;
}

}  // namespace deer
