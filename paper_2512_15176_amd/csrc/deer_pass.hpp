// The whole forward pass of one dense model as ONE persistent kernel (at most two 32-row tiles).
//
// Every phase of every layer (QKV projection, block attention, merge of its key-range splits, output
// projection, gate/up projection, down projection, then the LM head and the row statistics) is a loop over
// work items striped across the resident workgroups.  Phases are ordered by a split grid barrier: a
// workgroup ARRIVES when its share of a phase is stored, and WAITS for everybody's arrival only just before
// it reads the next phase's input.  Between the two it already requests the first weight fragments of its
// next GEMM item, which do not depend on any activation, so HBM keeps streaming while the dependency chain
// (partial sums -> last arrival -> epilogue -> barrier) resolves.
//
// Data that crosses workgroups inside the kernel (they may sit on XCDs with separate L2s):
//  - activation fragments live in per-layer buffers that are written once per pass, with agent-scope
//    (write-through) stores, and are only read after the barrier that follows; no cache can hold an older
//    copy of those lines, so they are read with plain loads and shared through L2 by the workgroups of an
//    XCD (an agent-scope load would fetch them from memory once per workgroup);
//  - the same holds for the K/V rows this pass appends: a layer's cache lines are first read in that
//    layer's attention phase;
//  - split-K partials, attention partials, the residual stream h, the sums of squares and the LM-head row
//    statistics are rewritten during the pass and use agent-scope loads and stores;
//  - weights, the prefix K/V rows, RoPE tables and row metadata were written by earlier kernels.
//
// Waiting is bounded: a workgroup that polls longer than the limit raises an error flag, after which nobody
// waits any more, the grid drains with meaningless results, and the host reports the failure.  The launch
// is cooperative, so all workgroups are resident and the limit is never reached in a healthy run.
#pragma once
#include "deer_kernels.hpp"

namespace deer {

// Barrier words (4 KB apart, so that they sit in different memory channels): the arrival counter, PASS_NF
// copies of the release flag (a workgroup polls copy blockIdx % PASS_NF; polling the counter itself would
// queue the arrivals behind hundreds of polls of the same line), and the error flag.
constexpr int PASS_NF = 8;
constexpr int PASS_SYNC_STRIDE = 1024;                              // words
constexpr int PASS_SYNC_WORDS = (PASS_NF + 3) * PASS_SYNC_STRIDE;
__host__ __device__ __forceinline__ int pass_flag_word(int f) { return (1 + f) * PASS_SYNC_STRIDE; }
__host__ __device__ __forceinline__ int pass_err_word() { return (1 + PASS_NF) * PASS_SYNC_STRIDE; }
__host__ __device__ __forceinline__ int pass_xcd_word() { return (2 + PASS_NF) * PASS_SYNC_STRIDE; }   // placement check failed

struct PassArgs {
    // model
    int L, d, Hq, Hkv, hd, F, V, n_qkv, kattn;
    float eps;
    const char *lw0; size_t layer_bytes, lo_qkv, lo_o, lo_gu, lo_d;
    const char *w_lm;
    uint16_t *kv_k, *kv_v; size_t kv_layer_stride, kv_seq_stride, kv_head_stride; int max_seq;
    // buffers
    RowMeta rm; const float2 *cs;
    float *h, *ssq, *part, *opart; int *counters;
    uint4 *xbase; size_t x_layer;     // per-layer activation fragments, (L + 1) layers of x_layer vectors
    // plan
    int nb;                                  // workgroups of the launch (the kernel never reads the launch
                                             // dimensions back from the dispatch arguments: that is a load from
                                             // the argument segment each time, on the critical path of a barrier)
    int ntiles, S_qkv, S_o, S_gu, S_d, NS;   // S > 0: that many equal K splits per column group;
    int stream_gu;                           // 1: the gate/up phase gives every workgroup an equal run of consecutive k-steps instead
    int allow_near;                          // 1: exchange inside an XCD's L2 where the placement check allows it
    float scale_log2e;
    int lm_on, lm_mt0, lm_stride, lm_tiles, k; float T; uint64_t seed;
    float *logits; RowStat *stat; RowResult *res;
    // synchronisation words (see PASS_SYNC_WORDS); counter and flags are zero before the launch
    unsigned *sync; unsigned spin_limit;
    // optional timeline: stamps[block][PASS_STAMPS] of the constant-rate clock, two per phase (input ready,
    // own items stored); null unless the host asked for it
    unsigned long long *stamps;
};
constexpr int PASS_STAMPS = 512;
__device__ __forceinline__ void stamp(const PassArgs &p, int &n) {
    if (p.stamps && threadIdx.x == 0 && n < PASS_STAMPS) p.stamps[(size_t)blockIdx.x * PASS_STAMPS + n] = wall_clock64();
    ++n;
}

// vectors (16 bytes) per tile of a fragment plane over `width` channels
__host__ __device__ __forceinline__ size_t plane_vecs(int width) { return (size_t)(width / 16) * 64; }
// per layer: X0 (input of QKV), Q, X1 (attention output), X2 (input of gate/up), X3 (SwiGLU output); hi and lo
__host__ __device__ __forceinline__ size_t pass_x_layer_vecs(int d, int kattn, int F, int ntiles) {
    return 2 * (size_t)ntiles * (2 * plane_vecs(d) + 2 * plane_vecs(kattn) + plane_vecs(F));
}
struct LayerX { uint4 *x0h, *x0l, *qh, *ql, *x1h, *x1l, *x2h, *x2l, *x3h, *x3l; };
__device__ __forceinline__ LayerX layer_x(const PassArgs &p, int l) {
    const size_t nd = p.ntiles * plane_vecs(p.d), nq = p.ntiles * plane_vecs(p.kattn), nf = p.ntiles * plane_vecs(p.F);
    LayerX x;
    x.x0h = p.xbase + (size_t)l * p.x_layer; x.x0l = x.x0h + nd;
    x.qh = x.x0l + nd; x.ql = x.qh + nq;
    x.x1h = x.ql + nq; x.x1l = x.x1h + nq;
    x.x2h = x.x1l + nq; x.x2l = x.x2h + nd;
    x.x3h = x.x2l + nd; x.x3l = x.x3h + nf;
    return x;
}

// Every thread has drained its stores of the phase (drain_vmem) before the workgroup is counted in.  The
// workgroup that completes the count releases the others by writing the epoch into the flag copies.
__device__ __forceinline__ void bar_arrive(const PassArgs &p, unsigned &epoch, int nb) {
    ++epoch;
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned old = __hip_atomic_fetch_add(p.sync, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old + 1u == epoch * (unsigned)nb) {
#pragma unroll
            for (int f = 0; f < PASS_NF; ++f)
                __hip_atomic_store(p.sync + pass_flag_word(f), epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// Returns when all workgroups have arrived `epoch` times.  Wave 0 polls its copy of the release flag.
__device__ __forceinline__ void bar_wait(const PassArgs &p, unsigned epoch) {
    if (epoch == 0) return;
    if ((threadIdx.x >> 6) == 0) {
        unsigned *err = p.sync + pass_err_word();
        const unsigned *flag = p.sync + pass_flag_word(blockIdx.x % PASS_NF);
        unsigned polls = 0;
        if (!__hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
            while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < epoch) {
                __builtin_amdgcn_s_sleep(1);
                if (++polls > p.spin_limit) { __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); break; }
                if ((polls & 63u) == 0 && __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) break;
            }
        }
    }
    __syncthreads();
    asm volatile("buffer_inv sc0" ::: "memory");   // drop this CU's cached copies of lines other workgroups rewrite
}

// ---- the sequence of GEMM items of one workgroup ------------------------------------------------
struct GemmDesc { const uint4 *W; int KS, S, ncg, stream; };   // stream: equal consecutive shares (S unused)
__device__ __forceinline__ GemmDesc phase_desc(const PassArgs &p, int l, int ph) {
    GemmDesc g;
    if (l >= p.L) {
        g.W = (const uint4 *)p.w_lm; g.KS = p.d / 16; g.S = 1; g.stream = 0; g.ncg = p.lm_on ? p.V / CG : 0;
        return g;
    }
    const char *lw = p.lw0 + (size_t)l * p.layer_bytes;
    g.stream = 0;
    if (ph == 0) { g.W = (const uint4 *)(lw + p.lo_qkv); g.KS = p.d / 16; g.S = p.S_qkv; g.ncg = p.n_qkv / CG; }
    else if (ph == 1) { g.W = (const uint4 *)(lw + p.lo_o); g.KS = p.kattn / 16; g.S = p.S_o; g.ncg = p.d / CG; }
    else if (ph == 2) { g.W = (const uint4 *)(lw + p.lo_gu); g.KS = p.d / 16; g.S = p.S_gu; g.stream = p.stream_gu; g.ncg = 2 * p.F / CG; }
    else { g.W = (const uint4 *)(lw + p.lo_d); g.KS = p.F / 16; g.S = p.S_d; g.ncg = p.d / CG; }
    return g;
}
// The workgroups form G groups of R; a group owns the column groups cg = gi (mod G) of every GEMM phase, the
// kv heads kvh = gi (mod G) of attention, and everything its members exchange with each other.  With the
// placement check passed, a group is the 32 workgroups of one XCD (G = 8, workgroup b sits on XCD b % 8) and
// that exchange stays in the XCD's L2; otherwise there is one group of all workgroups and the exchange goes
// through memory.
struct Grouping { int G, gi, R, r, nb; bool near; };
__device__ __forceinline__ Grouping make_grouping(bool near, int nb) {
    Grouping gr;
    gr.near = near;
    gr.nb = nb;
    if (near) { gr.G = 8; gr.gi = blockIdx.x & 7; gr.R = nb >> 3; gr.r = blockIdx.x >> 3; }
    else { gr.G = 1; gr.gi = 0; gr.R = nb; gr.r = blockIdx.x; }
    return gr;
}

// A piece of GEMM work: k-steps [kb, ke) of column group cg; it is the slot-th of np pieces of that group.
// Two ways to cut a group's share of a phase into pieces:
//  - S equal K splits per column group; piece index j = cgl + ncgl * s, striped over the group's workgroups;
//  - consecutive shares: the k-steps of the group's column groups are numbered column group by column group
//    and member r takes [r * u, (r + 1) * u), cut at column-group boundaries.  Every workgroup streams the
//    same number of bytes whatever the number of column groups.
struct Piece { int cg, kb, ke, slot, np; };
struct PieceIter { int pos, end, ncgl, u; };
__device__ __forceinline__ PieceIter piece_begin(const GemmDesc &g, const Grouping &gr) {
    PieceIter it;
    const int G = opaque_s(gr.G), R = opaque_s(gr.R);
    it.ncgl = (g.ncg - gr.gi + G - 1) / G;          // this group's column groups: cg = cgl * G + gi
    const int ncgl_max = (g.ncg + G - 1) / G;
    it.u = ((ncgl_max * g.KS + R - 1) / R + 7) / 8 * 8;
    if (g.stream) { it.pos = gr.r * it.u; it.end = min(it.ncgl * g.KS, it.pos + it.u); }
    else { it.pos = gr.r; it.end = it.ncgl * g.S; }
    return it;
}
__device__ __forceinline__ bool piece_valid(const PieceIter &it) { return it.pos < it.end; }
__device__ __forceinline__ Piece piece_at(const GemmDesc &g, const Grouping &gr, const PieceIter &it) {
    Piece pc;
    int cgl;
    const int KS = opaque_s(g.KS), u = opaque_s(it.u), ncgl = opaque_s(it.ncgl);
    if (g.stream) {
        cgl = it.pos / KS;
        pc.kb = it.pos - cgl * KS;
        pc.ke = min(KS, pc.kb + (it.end - it.pos));
        const int first = (cgl * KS) / u, last = ((cgl + 1) * KS - 1) / u;
        pc.slot = gr.r - first;
        pc.np = last - first + 1;
    } else {
        cgl = it.pos % ncgl;
        pc.slot = it.pos / ncgl;
        pc.np = g.S;
        const int per = (KS + g.S * 8 - 1) / opaque_s(g.S * 8) * 8;
        pc.kb = min(g.KS, pc.slot * per);
        pc.ke = min(g.KS, pc.kb + per);
    }
    pc.cg = cgl * gr.G + gr.gi;
    return pc;
}
__device__ __forceinline__ void piece_advance(const GemmDesc &g, const Grouping &gr, PieceIter &it, const Piece &pc) {
    if (g.stream) it.pos += pc.ke - pc.kb;
    else it.pos += gr.R;
}
// k-steps [ks0, ks1) of wave w inside a piece
__device__ __forceinline__ void wave_slice(const Piece &pc, int w, int &ks0, int &ks1) {
    const int per = (pc.ke - pc.kb + 7) >> 3;
    ks0 = pc.kb + w * per;
    ks1 = min(pc.ke, ks0 + per);
}

// Requests the first D k-steps of weight fragments of a piece (they do not depend on any activation, so
// this happens before the wait for the phase's input).  Every register of wb is overwritten: k-steps past
// the wave's slice repeat an in-range address and are not used.
template <int D>
__device__ __forceinline__ void w_issue(uint4 (&wb)[D][4], const GemmDesc &g, const Piece &pc, int w, int lane) {
    int ks0, ks1;
    wave_slice(pc, w, ks0, ks1);
    const uint4 *wp = g.W + ((size_t)(pc.cg * 4) * g.KS) * 64 + lane;
    const size_t wstride = (size_t)g.KS * 64;
#pragma unroll
    for (int dd = 0; dd < D; ++dd) {
        const int ks = min(ks0 + dd, g.KS - 1);
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) wb[dd][nb] = ld16_stream(wp + nb * wstride + (size_t)ks * 64);
    }
}

// The GEMM code below exists once per kernel and serves every phase: the epilogue kind is a run-time
// value.  (One copy per kind, as templates give, makes the kernel larger than the instruction cache, and
// every phase of every layer then fetches its code from memory again.)
__device__ __forceinline__ void pass_epilogue(int epi, const GemmArgs &a, GemmSmem &sm, const float (&hreg)[8], int cg, int ct) {
    float *rstd = sm.rstd + 32 * ct;   // filled at the start of the piece
    if (epi == EPI_QKV) run_epilogue<EPI_QKV, true, true>(a, sm.tile, rstd, sm.red, hreg, cg, ct);
    else if (epi == EPI_RESID) run_epilogue<EPI_RESID, true, true>(a, sm.tile, rstd, sm.red, hreg, cg, ct);
    else if (epi == EPI_SWIGLU) run_epilogue<EPI_SWIGLU, true, true>(a, sm.tile, rstd, sm.red, hreg, cg, ct);
    else run_epilogue<EPI_LMHEAD, true, true>(a, sm.tile, rstd, sm.red, hreg, cg, ct);
}

// Sums the S partial tiles of column group cg in order s = 0..S-1 and runs the epilogue (as gemm_finish).
template <int MT>
__device__ __forceinline__ void pass_finish(int epi, const GemmArgs &a, GemmSmem &sm, int cg, int S) {
    const int tidx = opaque_tid();
    const int N = a.N;
    float hreg[8];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int ct = mt;
        if (mt > 0) __syncthreads();
        if (epi == EPI_RESID) resid_prefetch<true>(a, hreg, cg, a.mt0 + ct * a.mt_stride);
        const size_t sstride = (size_t)a.rows_total * N;
        const float *pp[4];
        float2 v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = tidx + 512 * i;
            pp[i] = a.part + ((size_t)ct * 32 + (e >> 6)) * N + (size_t)cg * CG + (e & 63) * 2;
            v[i] = make_float2(0.f, 0.f);
        }
        for (int s0 = 0; s0 < S; s0 += 8) {   // 8 splits x 4 elements of loads in flight, summed in order
            float2 pv[8][4];
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i) pv[u][i] = ld_x2(pp[i] + (size_t)min(s0 + u, S - 1) * sstride, a.near != 0);
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (s0 + u < S) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) { v[i].x += pv[u][i].x; v[i].y += pv[u][i].y; }
                }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = tidx + 512 * i;
            float *tp = sm.tile + (e >> 6) * RED_STRIDE + (e & 63) * 2;
            tp[0] = v[i].x; tp[1] = v[i].y;
        }
        __syncthreads();
        pass_epilogue(epi, a, sm, hreg, cg, ct);
    }
}

// One piece of GEMM work.  wb holds the piece's first D weight k-steps, requested by gemm_phase.
template <int MT, int D>
__device__ __forceinline__ void gemm_item(const GemmArgs &a, int epi, GemmSmem &sm, const Piece &pc,
                                          uint4 (&wb)[D][4]) {
    const int tidx = opaque_tid();
    const int w = __builtin_amdgcn_readfirstlane(tidx >> 6), lane = tidx & 63;
    const int N = a.N, KS = a.KS, S = pc.np, cg = pc.cg, s = pc.slot;
    int ks0, ks1;
    wave_slice(pc, w, ks0, ks1);
    // The RMSNorm factors of the input rows only depend on the previous phase: their loads travel with the
    // first activation loads instead of forming a round trip of their own in the epilogue.
    // Requested here (at most 64 groups: 4 values per thread, 16 threads per row), summed after the k-loop.
    float ssqv[MT][4];
    if (epi != EPI_RESID) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const float *sp = a.ssq_in + (size_t)((a.mt0 + mt * a.mt_stride) * 32 + (tidx >> 4)) * a.ncg_in;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int gi = (tidx & 15) + 16 * i;
                ssqv[mt][i] = ldf<true>(sp + min(gi, a.ncg_in - 1));
            }
        }
    }

    f32x16 acc[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nb][r] = 0.f;

    const uint4 *wp = a.W + ((size_t)(cg * 4) * KS) * 64 + lane;
    const size_t wstride = (size_t)KS * 64;
    const uint4 *xh[MT], *xl[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const size_t tl = (size_t)(a.mt0 + mt * a.mt_stride);
        xh[mt] = a.Xhi + tl * KS * 64 + lane;
        xl[mt] = a.Xlo + tl * KS * 64 + lane;
    }
    // W fragments run D k-steps ahead (HBM latency), activation fragments DX k-steps ahead (L2 latency)
    constexpr int DX = (D < 4) ? D : 4;
    uint4 xhb[DX][MT], xlb[DX][MT];
#pragma unroll
    for (int dd = 0; dd < DX; ++dd)
        if (ks0 + dd < ks1) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) { xhb[dd][mt] = xh[mt][(size_t)(ks0 + dd) * 64]; xlb[dd][mt] = xl[mt][(size_t)(ks0 + dd) * 64]; }
        }
    for (int kb = ks0; kb < ks1; kb += D) {
#pragma unroll
        for (int dd = 0; dd < D; ++dd) {
            const int ks = kb + dd;
            if (ks < ks1) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb) {
                        acc[mt][nb] = mfma32(xhb[dd % DX][mt], wb[dd][nb], acc[mt][nb]);
                        acc[mt][nb] = mfma32(xlb[dd % DX][mt], wb[dd][nb], acc[mt][nb]);
                    }
                const int kn = ks + D, kx = ks + DX;
                if (kn < ks1) {
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb) wb[dd][nb] = ld16_stream(wp + nb * wstride + (size_t)kn * 64);
                }
                if (kx < ks1) {
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) { xhb[dd % DX][mt] = xh[mt][(size_t)kx * 64]; xlb[dd % DX][mt] = xl[mt][(size_t)kx * 64]; }
                }
            }
        }
    }


    __syncthreads();   // the previous piece's epilogue has finished with the tile, the scratch and sm.rstd
    if (epi != EPI_RESID) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float sq = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i) sq += ((tidx & 15) + 16 * i < a.ncg_in) ? ssqv[mt][i] : 0.f;
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) sq += shx(sq, off);
            if ((tidx & 15) == 0) sm.rstd[32 * mt + (tidx >> 4)] = rsqrtf(sq / (float)a.d_in + a.eps);
        }
    }
    float hreg[8];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int ct = mt;
        if (mt > 0) __syncthreads();
        if (epi == EPI_RESID && S == 1) resid_prefetch<true>(a, hreg, cg, a.mt0 + ct * a.mt_stride);
        reduce_waves_to_tile(acc[mt], sm.red, sm.tile, w, lane);
        if (S == 1) {
            pass_epilogue(epi, a, sm, hreg, cg, ct);
        } else {
            float *out = a.part + ((size_t)s * a.rows_total + (size_t)ct * 32) * N + (size_t)cg * CG;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = tidx + 512 * i;
                const int row = e >> 6, c2 = (e & 63) * 2;
                const float *tp = sm.tile + row * RED_STRIDE + c2;
                st_agent2(out + (size_t)row * N + c2, tp[0], tp[1]);
            }
        }
    }
    if (S == 1) {
        drain_vmem();   // the epilogue's stores are performed before the workgroup arrives at the barrier
    } else {
        const bool last = arrive_last(a.counters + cg, S, &sm.last, a.near != 0);   // drains this thread's stores first
        if (last) { pass_finish<MT>(epi, a, sm, cg, S); drain_vmem(); }
    }
}

// per LM row: merge the per-group statistics (512 threads; same result as k_rowstat_final)
__device__ __forceinline__ void rowstat_row(const RowStat *stat, int ncg_v, float T, RowResult *res, int row, float *scr) {
    const int tidx = opaque_tid();
    float *sm_ = scr; int *si = (int *)(scr + 512); float *sg = scr + 1024; int *sgi = (int *)(scr + 1536); float *ss = scr + 2048;
    const RowStat *p = stat + (size_t)row * ncg_v;
    float m = -INFINITY, gm = -INFINITY; int idx = 0x7fffffff, gidx = 0x7fffffff;
    for (int g = tidx; g < ncg_v; g += 512) {
        argmax_merge(m, idx, ldf<true>(&p[g].m), __hip_atomic_load(&p[g].idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        argmax_merge(gm, gidx, ldf<true>(&p[g].gm), __hip_atomic_load(&p[g].gidx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    }
    sm_[tidx] = m; si[tidx] = idx; sg[tidx] = gm; sgi[tidx] = gidx;
    __syncthreads();
    for (int off = 256; off > 0; off >>= 1) {
        if (tidx < off) {
            argmax_merge(sm_[tidx], si[tidx], sm_[tidx + off], si[tidx + off]);
            argmax_merge(sg[tidx], sgi[tidx], sg[tidx + off], sgi[tidx + off]);
        }
        __syncthreads();
    }
    const float M = sm_[0];
    float se = 0.f;
    if (T > 0.f) {
        const float invT = 1.f / T;
        for (int g = tidx; g < ncg_v; g += 512) se += ldf<true>(&p[g].sumexp) * expf((ldf<true>(&p[g].m) - M) * invT);
    }
    ss[tidx] = se;
    __syncthreads();
    for (int off = 256; off > 0; off >>= 1) {
        if (tidx < off) ss[tidx] += ss[tidx + off];
        __syncthreads();
    }
    if (tidx == 0) {
        RowResult r;
        const int V = ncg_v * CG;
        r.argmax = (si[0] >= 0 && si[0] < V) ? si[0] : 0;
        r.zmax = M;
        if (T > 0.f) { r.sample = (sgi[0] >= 0 && sgi[0] < V) ? sgi[0] : 0; r.lse = M / T + logf(ss[0]); }
        else { r.sample = r.argmax; r.lse = 0.f; }
        res[row] = r;
    }
    __syncthreads();
}

union PassSmem {
    GemmSmem g;
    AttnSmem at;
};

template <int MT, int D>
__device__ __forceinline__ void gemm_phase(const PassArgs &p, GemmArgs &a, int epi, GemmSmem &sm, const GemmDesc &g,
                                           const Grouping &gr, unsigned &epoch, int &ns) {
    a.W = g.W; a.KS = g.KS; a.S = g.S; a.N = g.ncg * CG; a.near = (gr.near && (p.allow_near & 1)) ? 1 : 0; a.h_near = (gr.near && (p.allow_near & 2)) ? 1 : 0;
    const int tidx = opaque_tid();
    const int w = __builtin_amdgcn_readfirstlane(tidx >> 6), lane = tidx & 63;
    // The first piece's first weights travel while the previous phase's dependency chain resolves; a workgroup
    // without a piece makes a harmless in-range request so that wb is defined on every path.
    uint4 wb[D][4];
    PieceIter it = piece_begin(g, gr);
    Piece pc = piece_valid(it) ? piece_at(g, gr, it) : Piece{0, 0, min(g.KS, 8), 0, 1};
    w_issue<D>(wb, g, pc, w, lane);
    bar_wait(p, epoch);   // the phase's input is complete
    stamp(p, ns);
    while (piece_valid(it)) {
        gemm_item<MT, D>(a, epi, sm, pc, wb);
        piece_advance(g, gr, it, pc);
        if (piece_valid(it)) { pc = piece_at(g, gr, it); w_issue<D>(wb, g, pc, w, lane); }
    }
    stamp(p, ns);
    bar_arrive(p, epoch, gr.nb);
}

template <int HD, int MT>
__global__ __launch_bounds__(512) void k_pass(const PassArgs p) {
    __shared__ __attribute__((aligned(16))) PassSmem smem;
    GemmSmem &sm = smem.g;
    constexpr int D = (MT == 1) ? 4 : 2;   // weight k-steps in flight per wave
    unsigned epoch = 0;
    int ns = 0;
    const int ntiles = p.ntiles, d = p.d, ncg_d = d / CG;
    // constants of the pass that the attention phase of every layer needs: per tile its sequence and per
    // query row its key limit.  Kept in LDS: registers that live through the whole kernel end up in scratch
    // memory, and a reload from there is a full memory round trip on the critical path of a phase.
    __shared__ int s_lim[64], s_seq[2];
    if (threadIdx.x < 64) s_lim[threadIdx.x] = p.rm.limit[min((int)threadIdx.x, ntiles * 32 - 1)];
    if (threadIdx.x < 2) s_seq[threadIdx.x] = p.rm.tile_seq[min((int)threadIdx.x, ntiles - 1)];
    __syncthreads();
    GemmArgs base{};
    base.part = p.part; base.counters = p.counters;
    base.mt0 = 0; base.mt_stride = 1; base.rows_total = ntiles * 32;
    base.ssq_in = p.ssq; base.ncg_in = ncg_d; base.d_in = d; base.eps = p.eps;
    base.cs = p.cs; base.rm = p.rm;
    base.Hq = p.Hq; base.Hkv = p.Hkv; base.hd = p.hd;
    base.h = p.h; base.ssq_out = p.ssq; base.F = p.F;


    // Placement check: the in-XCD exchange needs workgroup b on XCD b % 8, eight XCDs with equally many
    // workgroups.  Every workgroup compares its XCC id; one barrier later all of them know the outcome.
    bool near = false;
    const int nb = opaque_s(p.nb);
    if (p.allow_near && (nb & 7) == 0) {
        const unsigned xcc = __builtin_amdgcn_s_getreg((4 - 1) << 11 | 20) & 15u;   // HW_REG_XCC_ID, 4 bits
        if (xcc != (blockIdx.x & 7u) && threadIdx.x == 0)
            __hip_atomic_store(p.sync + pass_xcd_word(), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        drain_vmem();
        bar_arrive(p, epoch, nb);
        bar_wait(p, epoch);
        near = __hip_atomic_load(p.sync + pass_xcd_word(), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u;
    }
    const Grouping gr = make_grouping(near, nb);

    // all GEMM phases of all layers run through the one copy of the GEMM code in this loop
    const int n_phases = 4 * p.L + ((MT == 1 && p.lm_on) ? 1 : 0);
#pragma unroll 1
    for (int gph = 0; gph < n_phases; ++gph) {
        const int l = gph >> 2, ph = gph & 3;
        const LayerX x = layer_x(p, l), xn = layer_x(p, l + 1);
        uint16_t *Kl = p.kv_k + (size_t)l * p.kv_layer_stride, *Vl = p.kv_v + (size_t)l * p.kv_layer_stride;
        GemmArgs a = base;
        int epi;
        if (l == p.L) {          // LM head (single-tile passes; two-tile passes run it below on one tile)
            epi = EPI_LMHEAD;
            a.Xhi = x.x0h; a.Xlo = x.x0l;
            a.mt0 = p.lm_mt0; a.mt_stride = p.lm_stride;
            a.k = p.k; a.T = p.T; a.seed = p.seed; a.stat = p.stat; a.ncg_v = p.V / CG; a.logits = p.logits;
        } else if (ph == 0) {    // fused QKV projection, RoPE, cache write
            epi = EPI_QKV;
            a.Xhi = x.x0h; a.Xlo = x.x0l; a.qhi = x.qh; a.qlo = x.ql;
            a.kv = KvView{Kl, Vl, p.kv_seq_stride, p.kv_head_stride, p.max_seq};
        } else if (ph == 1) {    // output projection + residual
            epi = EPI_RESID;
            a.Xhi = x.x1h; a.Xlo = x.x1l; a.xhi_out = x.x2h; a.xlo_out = x.x2l;
        } else if (ph == 2) {    // gate/up projection + SwiGLU
            epi = EPI_SWIGLU;
            a.Xhi = x.x2h; a.Xlo = x.x2l; a.ahi = x.x3h; a.alo = x.x3l;
        } else {                 // down projection + residual
            epi = EPI_RESID;
            a.Xhi = x.x3h; a.Xlo = x.x3l; a.xhi_out = xn.x0h; a.xlo_out = xn.x0l;
        }
        gemm_phase<MT, D>(p, a, epi, sm, phase_desc(p, l, ph), gr, epoch, ns);
        if (ph != 0 || l == p.L) continue;

        // block attention: one (tile, kv head, key-range split) item per workgroup at a time
        bar_wait(p, epoch);
        stamp(p, ns);
        // a group's items: (tile, its kv heads kvh = kvl * G + gi, split); all splits of a kv head stay in the group
        const int nkvl = (p.Hkv - gr.gi + gr.G - 1) / opaque_s(gr.G);
        const int n_items = ntiles * nkvl * p.NS;
        for (int j = gr.r; j < n_items; j += gr.R) {
            const int NSo = opaque_s(p.NS), nkvo = opaque_s(nkvl);
            const int split = j % NSo, kvh = ((j / NSo) % nkvo) * gr.G + gr.gi, t = j / (NSo * nkvo);
            attn_item<HD>(x.qh, x.ql, Kl, Vl, p.kv_seq_stride, p.kv_head_stride, p.max_seq, s_seq[t],
                          s_lim[t * 32 + (opaque_tid() & 31)], p.opart, p.Hq, p.Hkv, p.NS, p.scale_log2e, x.x1h, x.x1l, smem.at, kvh, split, t);
        }
        drain_vmem();
        stamp(p, ns);
        bar_arrive(p, epoch, nb);
        if (p.NS > 1) {
            constexpr int HT = HD / 32;
            const int Gq = p.Hq / opaque_s(p.Hkv);
            const int n = ntiles * nkvl * Gq * HT * 2;
            bar_wait(p, epoch);
            stamp(p, ns);
            const int mt_ = opaque_tid(), w = __builtin_amdgcn_readfirstlane(mt_ >> 6), lane = mt_ & 63;
            for (int j = w * gr.R + gr.r; j < n; j += 8 * gr.R) {
                const int Gqo = opaque_s(Gq), nkvo = opaque_s(nkvl);
                const int hh = j & 1, tt = (j >> 1) % HT, gq = (j / (2 * HT)) % Gqo;
                const int kvh = ((j / (2 * HT * Gqo)) % nkvo) * gr.G + gr.gi, t = j / (2 * HT * Gqo * nkvo);
                attn_merge_item<HD>(p.opart, p.NS, p.Hq, p.scale_log2e, x.x1h, x.x1l, kvh * Gq + gq, t, tt, hh, lane, gr.near && (p.allow_near & 4));
            }
            drain_vmem();
            stamp(p, ns);
            bar_arrive(p, epoch, nb);
        }
    }
    if (p.lm_on) {
        if (MT != 1) {   // the LM head reads one tile
            const LayerX x = layer_x(p, p.L);
            GemmArgs a = base;
            a.Xhi = x.x0h; a.Xlo = x.x0l;
            a.mt0 = p.lm_mt0; a.mt_stride = p.lm_stride;
            a.k = p.k; a.T = p.T; a.seed = p.seed; a.stat = p.stat; a.ncg_v = p.V / CG; a.logits = p.logits;
            gemm_phase<1, D>(p, a, EPI_LMHEAD, sm, phase_desc(p, p.L, 0), gr, epoch, ns);
        }
        bar_wait(p, epoch);
        stamp(p, ns);
        for (int row = blockIdx.x; row < p.lm_tiles * p.k; row += nb)
            rowstat_row(p.stat, p.V / CG, p.T, p.res, row, sm.red);
        stamp(p, ns);
    }
}

}  // namespace deer
