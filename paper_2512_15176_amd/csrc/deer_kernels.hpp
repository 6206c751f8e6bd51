// Device code of libdeer: every step of the draft-verify iteration as HIP kernels for gfx950.
//
// Data layouts (all chosen for 64-lane wavefronts and the 32x32x16 bf16 MFMA):
//   * "fragment" layout of a [32 rows x K] operand tile: 16-byte vectors ordered [K/16][64 lanes],
//     lane l holding row (l % 32), k-indices 16*ks + 8*(l / 32) .. +8.  One wave-wide 16-byte load
//     is one MFMA operand.  Weights use it per 32-column block ([N/32][K/16][64][8], so a block's
//     whole K extent is one contiguous stream); activations use it per 32-row tile, as two planes
//     (hi, lo) with x ~= hi + lo in bf16, so that products against bf16 weights are exact to
//     ~2^-17 and accumulate in fp32.
//   * residual stream h: fp32 row-major [rows][d_model].
//   * K and V caches [layer][seq][kv_head] in blocks of 32 slots, each block in the fragment order of the
//     attention contractions (see k_cache_off / v_cache_off), bf16.
//   * a pass works on row tiles of 32; every tile belongs to one sequence; unused rows have
//     limit 0 and slot -1.
#pragma once
#include <hip/hip_runtime.h>
#include <type_traits>
#include <stdint.h>

namespace deer {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;   // a 16-byte operand fragment held in registers

constexpr int TILE_M = 32;       // rows per tile
constexpr int CG = 128;          // columns per column group (4 MFMA column blocks)
constexpr int RED_STRIDE = 136;  // padded LDS row stride (floats) of a 32x128 tile

// ------------------------------------------------------------------------------------------
// small helpers
// ------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

// fp32 -> bf16, round to nearest even (the hardware conversion)
__device__ __forceinline__ uint32_t f2bf(float f) {
    return (uint32_t)__builtin_bit_cast(unsigned short, (__bf16)f);
}
__device__ __forceinline__ float bf2f(uint32_t b) { return __uint_as_float(b << 16); }
// two floats -> packed bf16 pair (a in the low half)
__device__ __forceinline__ uint32_t f2bf2(float a, float b) {
    f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// x ~= hi + lo, both bf16
__device__ __forceinline__ void split_bf(float x, uint32_t &hi, uint32_t &lo) {
    hi = f2bf(x);
    lo = f2bf(x - bf2f(hi));
}

__device__ __forceinline__ uint4 pack8(const float *v) {
    return make_uint4(f2bf2(v[0], v[1]), f2bf2(v[2], v[3]), f2bf2(v[4], v[5]), f2bf2(v[6], v[7]));
}

__device__ __forceinline__ void pack8_split(const float *v, uint4 &hi, uint4 &lo) {
    uint32_t h[4], l[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        h[e] = f2bf2(v[2 * e], v[2 * e + 1]);
        l[e] = f2bf2(v[2 * e] - __uint_as_float(h[e] << 16), v[2 * e + 1] - __uint_as_float(h[e] & 0xffff0000u));
    }
    hi = make_uint4(h[0], h[1], h[2], h[3]);
    lo = make_uint4(l[0], l[1], l[2], l[3]);
}

__device__ __forceinline__ f32x16 mfma32(uint4 a, uint4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 mfma32(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 mfma32(u32x4 a, uint4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// A 16-byte load of data that is read exactly once per pass (weights, the prefix K/V rows): marked
// non-temporal so that the stream does not push activations, partial sums and the kernel's own
// instructions out of L2.
__device__ __forceinline__ uint4 ld16_stream(const uint4 *p) {
    const u32x4 v = __builtin_nontemporal_load((const u32x4 *)p);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// Hand-scheduled loads (used where the compiler's wait-count insertion would drain every outstanding
// load at a loop header): the load is issued here and its result may only be read after wait_loads<N>()
// (at most N younger loads still outstanding; loads return in order) followed by tie() on the register.
__device__ __forceinline__ void load16_async(u32x4 &dst, const void *p) {
    asm volatile("global_load_dwordx4 %0, %1, off" : "=&v"(dst) : "v"(p) : "memory");
}
// the same, marked non-temporal (data read once per pass: weights)
__device__ __forceinline__ void load16_stream_async(u32x4 &dst, const void *p) {
    asm volatile("global_load_dwordx4 %0, %1, off nt" : "=&v"(dst) : "v"(p) : "memory");
}
__device__ __forceinline__ void load4_async(float &dst, const void *p) {
    asm volatile("global_load_dword %0, %1, off" : "=&v"(dst) : "v"(p) : "memory");
}
__device__ __forceinline__ void tie(float &r) { asm volatile("" : "+v"(r)); }
// at most `steps` x PER loads may still be outstanding (steps <= 4)
template <int PER>
__device__ __forceinline__ void wait_steps(int steps);
// The same with agent scope: the load is served by memory, not by an L2 that may hold an older copy of a line
// another XCD has written since.
__device__ __forceinline__ void load16_agent_async(u32x4 &dst, const void *p) {
    asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(dst) : "v"(p) : "memory");
}
// A 16-byte agent-scope (write-through) store.  The wait states behind it keep the next instruction from
// overwriting the data registers while the store still reads them (a hazard the compiler covers for its own
// stores of more than 8 bytes, but cannot see inside an asm statement).
__device__ __forceinline__ void store16_agent(void *p, float a, float b, float c, float d) {
    u32x4 v = {__float_as_uint(a), __float_as_uint(b), __float_as_uint(c), __float_as_uint(d)};
    asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 2" ::"v"(p), "v"(v) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_loads() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
template <int PER>
__device__ __forceinline__ void wait_steps(int steps) {
    static_assert(4 * PER <= 63, "the counter has six bits");
    if (steps <= 0) wait_loads<0>();
    else if (steps == 1) wait_loads<PER>();
    else if (steps == 2) wait_loads<2 * PER>();
    else if (steps == 3) wait_loads<3 * PER>();
    else wait_loads<4 * PER>();
}
__device__ __forceinline__ void tie(u32x4 &r) { asm volatile("" : "+v"(r)); }

// Workgroup barrier for loops that keep direct-to-LDS loads in flight across it: __syncthreads() waits for every
// outstanding vector memory operation of the wave (its fence covers the LDS writes of those loads), which would
// empty the ring of staged buffers at every barrier.  This one waits only for the wave's LDS reads; the caller
// counts down the loads that must have landed with wait_loads<N>() first.
__device__ __forceinline__ void barrier_keep_loads() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// The thread index as a value the optimiser cannot trace back to the hardware register.  Lane-dependent
// indices and addresses derived from it are recomputed where they are used instead of being hoisted to the
// top of a long kernel and kept in registers (or spilled) across all of its phases.
__device__ __forceinline__ int opaque_tid() {
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));
    return t;
}

// Butterfly exchange with lane (lane ^ off).  The lane index is derived where it is used (see opaque_tid),
// never from a value computed once at the top of the kernel; blocks are whole wavefronts, so the low six
// bits of the thread index are the lane.
__device__ __forceinline__ int shx(int v, int off) {
    return __builtin_amdgcn_ds_bpermute(((opaque_tid() & 63) ^ off) << 2, v);
}
__device__ __forceinline__ float shx(float v, int off) { return __int_as_float(shx(__float_as_int(v), off)); }

// A uniform value the optimiser cannot trace: divisions by it are expanded where they stand.  (The reciprocal
// of a loop-invariant divisor is otherwise computed once at the top of the kernel, in a vector register that
// lives through the whole kernel, is spilled, and is reloaded from scratch memory at every use.)
__device__ __forceinline__ int opaque_s(int v) {
    asm volatile("" : "+s"(v));
    return v;
}

__device__ __forceinline__ void drain_vmem() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Row of the 32x32 MFMA result held in register r of a lane in half `half` (= lane / 32).
__device__ __forceinline__ int mfma_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// Index (in 16-byte vectors) of (row, k-octet) inside a fragment-layout tile with KS k-steps.
__device__ __forceinline__ size_t frag_vec(int row, int oct) { return (size_t)(oct >> 1) * 64 + row + 32 * (oct & 1); }

__device__ __forceinline__ uint64_t mix64(uint64_t z) {  // splitmix64 finaliser
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}
constexpr uint64_t GOLDEN = 0x9E3779B97F4A7C15ULL;
enum { TAG_DRAFT = 1, TAG_ACCEPT = 2, TAG_RESID = 3 };
__device__ __forceinline__ uint64_t row_key(uint64_t seed, uint64_t tag, uint64_t seq, uint64_t pos) {
    return mix64(mix64(seed + GOLDEN * tag) ^ ((seq << 40) + pos));
}
__device__ __forceinline__ float uniform01(uint64_t key, uint64_t idx) {  // (r + 0.5) / 2^23, r < 2^23
    uint64_t bits = mix64(key + GOLDEN * (idx + 1));
    return ((float)(uint32_t)(bits >> 41) + 0.5f) * (1.0f / 8388608.0f);
}
__device__ __forceinline__ float gumbel(uint64_t key, uint64_t idx) { return -logf(-logf(uniform01(key, idx))); }

// Split-K / split-KV partials cross workgroups that may sit on different XCDs (separate L2s).  They
// are written and read with agent-scope accesses, which are coherent without cache-wide
// write-backs or invalidates; the arrival counter is an agent-scope atomic.
__device__ __forceinline__ void st_agent2(float *p, float a, float b) {   // p 8-byte aligned
    unsigned long long u = ((unsigned long long)__float_as_uint(b) << 32) | (unsigned long long)__float_as_uint(a);
    __hip_atomic_store((unsigned long long *)p, u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_agent2(const float *p) {
    unsigned long long u = __hip_atomic_load((const unsigned long long *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_float2(__uint_as_float((unsigned)(u & 0xffffffffu)), __uint_as_float((unsigned)(u >> 32)));
}
// Called by every thread after its partial stores: waits for them, then one thread counts the block
// in.  Returns true in every thread of the block that arrived last (counter reset for the next use).
__device__ __forceinline__ bool arrive_last(int *cnt, int expected, int *s_flag) {
    // The thread's agent-scope stores must have been performed before the block is counted in.  A
    // workgroup-scope fence does not wait for vector memory, so the wait is explicit.
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0) {
        int old = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        int last = (old == expected - 1);
        if (last) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_flag = last;
    }
    __syncthreads();
    return *s_flag != 0;
}

// Stores of results that other workgroups read.  COH = true: agent-scope (write-through) stores, for data that
// crosses workgroups inside one kernel (they may sit on XCDs with separate L2s); COH = false: plain stores
// (producer and consumer are separated by a kernel boundary).
template <bool COH> __device__ __forceinline__ void stf(float *p, float v) {
    if (COH) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *p = v;
}
template <bool COH> __device__ __forceinline__ void sti(int *p, int v) {
    if (COH) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *p = v;
}
template <bool COH> __device__ __forceinline__ void st16(uint4 *p, uint4 v) {
    if (COH) {
        unsigned long long *q = (unsigned long long *)p;
        __hip_atomic_store(q, ((unsigned long long)v.y << 32) | v.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(q + 1, ((unsigned long long)v.w << 32) | v.z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
        *p = v;
    }
}
template <bool COH> __device__ __forceinline__ void st_u16(uint16_t *p, uint16_t v) {
    if (COH) __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    else *p = v;
}

// (value, index) max with lowest index on ties
__device__ __forceinline__ void argmax_merge(float &v, int &i, float v2, int i2) {
    if (v2 > v || (v2 == v && i2 < i)) { v = v2; i = i2; }
}

// ------------------------------------------------------------------------------------------
// weight repack: canonical [K][N_src] (fp32 or bf16) -> fragment layout, bf16
//   dest column n_dst = col_map(n_src):  plain offset (QKV concatenation) or gate/up interleave
//   (group of 128 columns = 64 gate channels followed by the same 64 up channels).
// ------------------------------------------------------------------------------------------
template <typename SrcT>
__device__ __forceinline__ uint32_t load_as_bf16(const SrcT *p);
template <>
__device__ __forceinline__ uint32_t load_as_bf16<float>(const float *p) { return f2bf(*p); }
template <>
__device__ __forceinline__ uint32_t load_as_bf16<uint16_t>(const uint16_t *p) { return *p; }

// mode 0: n_dst = n_src + col_off.  mode 1 (gate) / 2 (up): n_dst = (n_src/64)*128 + (mode-1)*64 + n_src%64
template <typename SrcT>
__global__ void k_repack(const SrcT *__restrict__ src, uint4 *__restrict__ dst, int K, int N_src, int KS_dst,
                         int mode, int col_off) {
    // one thread per (src column n, k-octet): reads 8 strided values, writes one 16-byte vector
    size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    int n = (int)(gid % N_src);
    size_t oct = gid / N_src;
    if (oct >= (size_t)K / 8) return;
    int n_dst = (mode == 0) ? n + col_off : (n / 64) * 128 + (mode - 1) * 64 + (n % 64);
    uint32_t v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = load_as_bf16<SrcT>(src + ((size_t)oct * 8 + e) * N_src + n);
    int nb = n_dst >> 5;
    size_t vec = ((size_t)nb * KS_dst) * 64 + frag_vec(n_dst & 31, (int)oct);
    dst[vec] = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
}

template <typename SrcT>
__global__ void k_convert_rows(const SrcT *__restrict__ src, uint16_t *__restrict__ dst, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = (uint16_t)load_as_bf16<SrcT>(src + i);
}

// Measurement aid: a plain read of n 16-byte vectors (grid-stride, four loads in flight per thread and trip), the rate
// of which is what "streaming at memory speed" means for a buffer of that size on this chip.  Nothing is written
// unless the data has one particular checksum (so that the loads cannot be dropped).
template <bool NT>
__global__ __launch_bounds__(512) void k_stream_read(const u32x4 *__restrict__ p, size_t n, uint32_t *out) {
    size_t i = (size_t)blockIdx.x * 512 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 512;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + 3 * stride < n; i += 4 * stride) {
        u32x4 v0, v1, v2, v3;
        if (NT) {
            v0 = __builtin_nontemporal_load(p + i); v1 = __builtin_nontemporal_load(p + i + stride);
            v2 = __builtin_nontemporal_load(p + i + 2 * stride); v3 = __builtin_nontemporal_load(p + i + 3 * stride);
        } else {
            v0 = p[i]; v1 = p[i + stride]; v2 = p[i + 2 * stride]; v3 = p[i + 3 * stride];
        }
        acc ^= v0 ^ v1 ^ v2 ^ v3;
    }
    for (; i < n; i += stride) acc ^= p[i];
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) out[0] = 1u;
}

__global__ void k_fill_u32(uint32_t *p, uint32_t v, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// ------------------------------------------------------------------------------------------
// per-sequence state and row metadata
// ------------------------------------------------------------------------------------------
struct SeqState {       // device arrays, one entry per sequence
    int *len;           // j: committed tokens
    int *dr_len;        // tokens in the drafter cache
    int *pending;       // x_j
    int *ing_n;         // committed tokens the drafter has not cached yet
    int *ing_tok;       // [B][32]
    int *finished;      // EOS seen
};

struct RowMeta {        // device arrays over the rows of a pass
    int *tok, *pos, *limit, *slot;   // [rows]; slot < 0: do not write K,V
    int *tile_seq;                   // [tiles]
};

// verify rows of sequence b: tile b; row i < nrows: [x_j, y^_1 .. y^_{nrows-1}] at positions j-1+i, with
// nrows = k, or k + 1 when the bonus token is on (the last draft is a row too)
// token ids that reach the embedding gather are forced into [0, vocab): drafts come from caller memory
__device__ __forceinline__ int safe_tok(int t, int vocab) { return (t < 0 || t >= vocab) ? 0 : t; }

// Rows of a verify or draft pass (Alg. 1: one pass per model and iteration).
//   verify: tile b = sequence b, nrows rows [x_j, y^_1 .. ]: row i at position j - 1 + i, causal over the cache.
//   draft: sequence b has tiles_per_seq tiles; tile 0 = k MASK rows at positions j..j+k-1 (they see the cache, the
//   ingested rows and every MASK row; their K,V land in slots past the cached length and are never kept); tile 1 = the
//   m not-yet-cached committed tokens, causal.  The first n_fixed block rows hold the tokens fixed[b][0 .. n_fixed)
//   instead of the MASK id (a partially filled block: a later pass of a multi-pass draft).
struct PassRows {
    int draft_pass;                  // 0: verify, 1: draft
    SeqState st;
    const int *tokens;               // verify: the draft tokens [B][k]; draft: the fixed tokens [B][k] (n_fixed > 0)
    int k, nrows, vocab;             // nrows: verify rows per sequence
    int mask_id, tiles_per_seq, n_fixed;
};
struct RowDesc { int tok, pos, slot, limit; };

__device__ __forceinline__ RowDesc pass_row(const PassRows &p, int tile, int r, int &b) {
    RowDesc d{0, 0, -1, 0};
    if (!p.draft_pass) {
        b = tile;
        if (r < p.nrows) {
            const int pos = p.st.len[b] - 1 + r;
            d.tok = safe_tok(r == 0 ? p.st.pending[b] : p.tokens[b * p.k + r - 1], p.vocab);
            d.pos = pos; d.slot = pos; d.limit = pos + 1;
        }
    } else {
        b = tile / p.tiles_per_seq;
        const int t = tile - b * p.tiles_per_seq;
        if (t == 0 && r < p.k) {
            const int j = p.st.len[b];
            d.tok = r < p.n_fixed ? safe_tok(p.tokens[b * p.k + r], p.vocab) : p.mask_id;
            d.pos = j + r; d.slot = j + r; d.limit = j + p.k;
        } else if (t == 1 && r < p.st.ing_n[b]) {
            const int dl = p.st.dr_len[b];
            d.tok = safe_tok(p.st.ing_tok[b * 32 + r], p.vocab);
            d.pos = dl + r; d.slot = dl + r; d.limit = dl + r + 1;
        }
    }
    return d;
}

// prefill pass: tile t holds desc[t].z rows of sequence desc[t].x, causal, at positions desc[t].y + r, whose token
// ids start at ids[desc[t].w].  A pass may hold tiles of several sequences (each sequence's rows in whole tiles).
__global__ void k_rows_prefill(RowMeta rm, const int *__restrict__ ids, const int4 *__restrict__ desc) {
    const int4 dsc = desc[blockIdx.x];
    const int r = threadIdx.x, row = blockIdx.x * 32 + r;
    if (r == 0) rm.tile_seq[blockIdx.x] = dsc.x;
    if (r < dsc.z) {
        rm.tok[row] = ids[dsc.w + r]; rm.pos[row] = dsc.y + r; rm.slot[row] = dsc.y + r; rm.limit[row] = dsc.y + r + 1;
    } else {
        rm.tok[row] = 0; rm.pos[row] = 0; rm.slot[row] = -1; rm.limit[row] = 0;
    }
}

// cos/sin of pos * theta_i, evaluated in double, stored fp32: cs[row][i] = (cos, sin)
__global__ void k_rope_table(const int *__restrict__ pos, const double *__restrict__ theta, float2 *__restrict__ cs,
                             int half, int rows) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rows * half) return;
    int row = idx / half, i = idx % half;
    double s, c;
    sincos((double)pos[row] * theta[i], &s, &c);
    cs[idx] = make_float2((float)c, (float)s);
}

// ------------------------------------------------------------------------------------------
// write a 32 x 128 fp32 tile (LDS, stride RED_STRIDE) into fragment layout (hi/lo) at k-columns
// k0 .. k0+127 of a tile with KS k-steps; 512 (row, octet) items over 256 threads
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void tile_to_frag(const float *tile, uint4 *xhi, uint4 *xlo, size_t tile_base_vec, int k0) {
    for (int item = threadIdx.x; item < 512; item += 256) {
        int row = item & 31, oct = item >> 5;
        uint4 hi, lo;
        pack8_split(tile + row * RED_STRIDE + oct * 8, hi, lo);
        size_t v = tile_base_vec + frag_vec(row, (k0 >> 3) + oct);
        xhi[v] = hi;
        xlo[v] = lo;
    }
}

// embedding gather of one (column group, tile): h[row] = E[tok[row]] (bf16 table), plus fragment planes and sums of
// squares; tok: the tile's 32 token ids (global memory or LDS); 256 threads
__device__ __forceinline__ void embed_tile(float *tile, const uint16_t *__restrict__ E, const int *tok, float *__restrict__ h,
                                           uint4 *__restrict__ xhi, uint4 *__restrict__ xlo, float *__restrict__ ssq, int d,
                                           int ncg, int ssq_sub, int cg, int t) {
    for (int e = threadIdx.x; e < 32 * CG; e += 256) {
        int row = e >> 7, col = e & 127;
        int grow = t * 32 + row;
        float v = bf2f(E[(size_t)tok[row] * d + cg * CG + col]);
        tile[row * RED_STRIDE + col] = v;
        h[(size_t)grow * d + cg * CG + col] = v;
    }
    __syncthreads();
    tile_to_frag(tile, xhi, xlo, (size_t)t * (d / 16) * 64, cg * CG);
    // sums of squares per row and column group, or (ssq_sub == 4) per 32-column block of it
    if (threadIdx.x < 32 * ssq_sub) {
        const int row = threadIdx.x & 31, blk = threadIdx.x >> 5, wdt = CG / ssq_sub;
        float s = 0.f;
        for (int c = 0; c < wdt; ++c) { float v = tile[row * RED_STRIDE + blk * wdt + c]; s += v * v; }
        ssq[(size_t)(t * 32 + row) * (ncg * ssq_sub) + cg * ssq_sub + blk] = s;
    }
}

__global__ __launch_bounds__(256) void k_embed(const uint16_t *__restrict__ E, const int *__restrict__ tok,
                                               float *__restrict__ h, uint4 *__restrict__ xhi, uint4 *__restrict__ xlo,
                                               float *__restrict__ ssq, int d, int ncg, int ssq_sub) {
    __shared__ float tile[32 * RED_STRIDE];
    embed_tile(tile, E, tok + blockIdx.y * 32, h, xhi, xlo, ssq, d, ncg, ssq_sub, blockIdx.x, blockIdx.y);
}

// The start of a draft or verify pass in one launch: every block works out its tile's rows (pass_row), then blocks
// x < ncg gather the embeddings of column group x, block x == ncg writes the row metadata and the tile's RoPE table.
// (Three launches of a few microseconds each left the GPU waiting for the host at the start of every pass.)
__global__ __launch_bounds__(256) void k_pass_begin(PassRows p, RowMeta rm, const uint16_t *__restrict__ E, float *__restrict__ h,
                                                    uint4 *__restrict__ xhi, uint4 *__restrict__ xlo, float *__restrict__ ssq,
                                                    int d, int ncg, int ssq_sub, const double *__restrict__ theta,
                                                    float2 *__restrict__ cs, int half) {
    __shared__ float tile[32 * RED_STRIDE];
    __shared__ int s_tok[32], s_pos[32];
    const int t = blockIdx.y;
    if (threadIdx.x < 32) {
        int b;
        const RowDesc r = pass_row(p, t, threadIdx.x, b);
        s_tok[threadIdx.x] = r.tok; s_pos[threadIdx.x] = r.pos;
        if (blockIdx.x == ncg) {
            const int row = t * 32 + threadIdx.x;
            rm.tok[row] = r.tok; rm.pos[row] = r.pos; rm.slot[row] = r.slot; rm.limit[row] = r.limit;
            if (threadIdx.x == 0) rm.tile_seq[t] = b;
        }
    }
    __syncthreads();
    if (blockIdx.x < ncg) {
        embed_tile(tile, E, s_tok, h, xhi, xlo, ssq, d, ncg, ssq_sub, blockIdx.x, t);
    } else {
        for (int idx = threadIdx.x; idx < 32 * half; idx += 256) {
            const int row = idx / half, i = idx - row * half;
            double sn, c;
            sincos((double)s_pos[row] * theta[i], &sn, &c);
            cs[(size_t)(t * 32 + row) * half + i] = make_float2((float)c, (float)sn);
        }
    }
}

// ------------------------------------------------------------------------------------------
// weight-streaming GEMM for short row counts with the layer's elementwise work fused behind it
//   y[i][n] = sum_k x[i][k] W[k][n]  for MT row tiles of 32 and one group of 128 columns per block.
//   grid: x = column group, y = split s of the K range, z = group of MT row tiles.
//   block: 8 waves; wave w streams k-slice (s*8 + w) of 8*S for all 4 column blocks of the group
//   (one activation fragment pair feeds 4 weight fragments); the 8 waves are summed through LDS in a
//   fixed tree.  S == 1: the epilogue runs on the tile in LDS.  S > 1: the tile goes to a partial
//   buffer and the block that arrives last at the group's counter sums the S partials in order
//   s = 0..S-1 and runs the epilogue, so results do not depend on arrival order.
//   Tiles of the launch: tile(ct) = mt0 + ct * mt_stride, ct = z*MT + mt.
// ------------------------------------------------------------------------------------------
enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LMHEAD = 3, EPI_ROUTER = 4 };

struct KvView {
    uint16_t *k, *vt;                                  // layer base already applied
    size_t seq_stride, head_stride;                    // elements
    int max_seq;
};

// Both caches are stored per (sequence, kv head) in blocks of 32 slots (one key tile), and inside a block in the
// order the attention kernels' MFMA operands want them: head_dim / 16 fragments of 64 lanes x 8 elements, so that
// a wave reads a fragment as one contiguous 1 KB and every cache line it touches is used whole.
//   K block, fragment s (k-step: elements 16 s .. 16 s + 15): lane (operand row r, half) holds elements
//   16 s + 8 half .. + 7 of the key whose operand row is r.  Operand rows are a permutation of the keys that gives
//   each lane of the S^T result 16 consecutive keys: key = 16 * bit2(r) + 4 * (r >> 3) + (r & 3).
//   V^T block, fragment (O^T tile tt, s2): lane (channel c = 32 tt + (lane & 31), half) holds keys
//   16 half + 8 s2 .. + 7 of channel c.
__device__ __forceinline__ int key_operand_row(int key) { return (key & 3) | (((key >> 4) & 1) << 2) | (((key >> 2) & 3) << 3); }
// element offset of octet `oct` (8 elements of head_dim) of slot `slot` inside a (sequence, kv head) K region
__device__ __forceinline__ size_t k_cache_off(int slot, int oct, int hd) {
    return ((size_t)(slot >> 5) * (hd >> 4) + (oct >> 1)) * 512 + ((oct & 1) * 32 + key_operand_row(slot & 31)) * 8;
}
// element offset of channel c of slot `slot` inside a (sequence, kv head) V^T region
__device__ __forceinline__ size_t v_cache_off(int slot, int c, int hd) {
    const int kk = slot & 31;
    return ((size_t)(slot >> 5) * (hd >> 4) + (c >> 5) * 2 + ((kk >> 3) & 1)) * 512 + ((kk >> 4) * 32 + (c & 31)) * 8 + (kk & 7);
}

struct RowStat {   // per (row, column group) partial over 128 vocabulary entries
    float m; int idx;        // max logit, its index (lowest on ties)
    float sumexp;            // sum exp(z/T - m/T)  (T > 0)
    float gm; int gidx;      // max of z/T + Gumbel, its index (T > 0)
};

// A load whose data nobody wants: it pulls a line into the L2.  The data goes to LDS (lane l's 16 bytes land at
// sink + 16 l: 1 KB per wave that the workgroup no longer needs), not to registers: a register that waits for a load
// has to be kept away from the compiler's allocator until the data is back, and nothing in the language does that
// across branches and loops.  The caller ends with wait_loads<0>(): the LDS must still be the workgroup's when the data
// arrives.
__device__ __forceinline__ void load16_discard(void *sink, const void *p) {
    asm volatile("; fetch ahead");
    __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)p,
                                     (void __attribute__((address_space(3))) *)sink, 16, 0, 0);
}

// What the NEXT launch of the stream will read first, for workgroups of this launch that have nothing left to do:
// they pull it into their XCD's L2 while the launch's last workgroups finish (memory is idle then), so that the next
// launch's first k-steps hit there.  Workgroup ids 8 apart share an XCD in both launches; workgroup j of this launch
// fetches for workgroup j of the next.
//   narrow_nb == 0 (k_gemm's grid order): next-launch workgroup j works on column group j % ncg and K split j / ncg;
//     fetched: the first `span` bytes of the split's K range in each of the group's four 32-column blocks.
//   narrow_nb = NB > 0 (k_gemm_narrow's order): j = 8 * ((p / 8) * Z + z) + p % 8 is row tile z of the group p of NB
//     blocks, all of K; the Z workgroups of a group read the same (contiguous) NB * block_bytes: part z of Z is fetched.
struct NextWeights {
    const char *base;          // the next launch's weight matrix, fragment layout; null: nothing to fetch
    int nwg, ncg;              // its workgroups and column groups (narrow: groups of NB blocks)
    int span;                  // bytes fetched per 32-column block, from the start of the split's K range
    long long block_bytes;     // one 32-column block: KS * 1024
    long long split_bytes;     // a split's K range within a block
    int narrow_nb, Z;
};

// lds: 8 KB of LDS the workgroup is done with
__device__ __forceinline__ void prefetch_next(const NextWeights &nx, void *lds) {
    if (!nx.base) return;
    // one next-launch workgroup per workgroup and no more: what is fetched must be back before this launch can end
    const int lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const int tid = opaque_tid();
    char *sink = (char *)lds + (__builtin_amdgcn_readfirstlane(tid >> 6) << 10);
    if (lin < nx.nwg && nx.narrow_nb > 0) {
        const int q8 = lin >> 3, z = q8 % nx.Z, grp = 8 * (q8 / nx.Z) + (lin & 7);
        if (grp < nx.ncg) {
            const int total = nx.narrow_nb * (int)nx.block_bytes;             // the group's blocks are adjacent
            const int part = ((total / 16 + nx.Z - 1) / nx.Z) * 16;
            const int end = min(total, (z + 1) * part);
            const char *p0 = nx.base + (long long)grp * total;
            for (int o = z * part + tid * 16; o < end; o += 512 * 16) load16_discard(sink, p0 + o);
        }
    } else if (lin < nx.nwg) {
        const int j = lin;
        const int cg = j % nx.ncg, sp = j / nx.ncg;
        const long long s_off = sp * nx.split_bytes;
        const int len = (int)min((long long)nx.span, nx.block_bytes - s_off);   // stays inside the block
        const char *p0 = nx.base + (long long)cg * 4 * nx.block_bytes + s_off + tid * 16;
        for (int nb = 0; nb < 4; ++nb)
            for (int o = tid * 16; o < len; o += 512 * 16) load16_discard(sink, p0 + nb * nx.block_bytes + (o - tid * 16));
    }
    wait_loads<0>();
}

// The same for the per-head attention launch that follows a QKV projection: its workgroups on XCD x work on kv head
// x % Hkv (Hkv divides 8; one sequence), so this launch's idle workgroups on XCD x pull that head's old K and V^T blocks
// — whole key tiles that this launch does not write — into its L2.
__device__ __forceinline__ void prefetch_kv(const uint16_t *k, const uint16_t *vt, size_t head_stride, int Hkv, int bytes, void *lds) {
    if (bytes <= 0) return;
    const int lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const int nlin = gridDim.x * gridDim.y * gridDim.z;
    const int per_x = (nlin - (lin & 7) + 7) >> 3;
    const int tid = opaque_tid();
    const size_t head = (size_t)((lin & 7) % Hkv) * head_stride;
    const char *kb = (const char *)(k + head), *vb = (const char *)(vt + head);
    char *sink = (char *)lds + (__builtin_amdgcn_readfirstlane(tid >> 6) << 10);
    for (int o = ((lin >> 3) * 512 + tid) * 16; o < bytes; o += per_x * 8192) {   // the host bounds `bytes`: a few trips
        load16_discard(sink, kb + o);
        load16_discard(sink, vb + o);
    }
    wait_loads<0>();
}

struct GemmArgs {
    NextWeights nx;
    int kv_fetch_bytes;   // QKV launch before a per-head attention launch over one sequence: bytes of each kv head's K (and V^T) blocks to pull in, or 0
    const uint4 *W, *Xhi, *Xlo;
    float *part; int *counters;
    int N, KS, S, mt0, mt_stride, rows_total;
    // RMSNorm of the GEMM input rows: rstd from per-group sums of squares (QKV, SWIGLU, LMHEAD)
    const float *ssq_in; int ncg_in, d_in; float eps;
    // QKV: RoPE, Q fragments, cache writes
    const float2 *cs; RowMeta rm; uint4 *qhi, *qlo; KvView kv; int Hq, Hkv, hd;
    // RESID: h += y, new fragments and sums of squares of h
    float *h; uint4 *xhi_out, *xlo_out; float *ssq_out;
    int ssq_sub;   // 1: one sum of squares per row and 128-column group; 4: one per 32-column block (narrow launches)
    // SWIGLU: activation fragments over F channels
    uint4 *ahi, *alo; int F;
    // LMHEAD: logits, per-group row statistics
    int k; float *logits; float T; uint64_t seed; RowStat *stat; int ncg_v;
    int draw;   // T > 0: also the Gumbel-max of the perturbed logits (a pass that samples its rows' tokens)
    unsigned long long *stamps;   // debugging: [workgroup][8] device-clock stamps of this launch, or null
    int k_lo;   // rows below k_lo keep the logits and statistics of an earlier pass (multi-pass draft)
    // ROUTER: top-k of softmax over n_experts (<= 128), renormalised
    int n_experts, top_k; int *route_e; float *route_w;
    int route_spread;   // 0: the model's routing; layer + 1: synthetic uniform routing (benchmarks of random-init mixtures)
};

// rstd[row] = rsqrt(sum_g ssq[row][g] / d + eps) for the 32 rows of a tile, into LDS.  512 threads: 16 per
// row, each sums the groups g = j, j + 16, .. in order, then a fixed butterfly over the 16 partial sums.
template <bool COH>
__device__ __forceinline__ void tile_rstd(const float *ssq, float *rstd, int grow0, int ncg, int d, float eps) {
    const int tidx = opaque_tid();
    const int row = tidx >> 4, j = tidx & 15;
    const float *p = ssq + (size_t)(grow0 + row) * ncg;
    float s = 0.f;
    for (int g = j; g < ncg; g += 16) s += p[g];
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) s += shx(s, off);
    if (j == 0) rstd[row] = rsqrtf(s / (float)d + eps);
}

// QKV epilogue: RMSNorm scale, RoPE, Q -> fragment planes per head, K -> cache, V -> transposed cache
// The tile holds columns cg * WIDTH .. + WIDTH - 1 with row stride STRIDE.  WIDTH is a multiple of head_dim, so that
// a head, and with it every rotation pair, lies inside one tile.
// pre (optional): what qkv_prefetch loaded for this thread's item while the tile was still being summed.
constexpr int QKV_PRE = 18;   // 8 (cos, sin) pairs, the row's cache slot, the tile's sequence
template <bool COH, int WIDTH = CG, int STRIDE = RED_STRIDE, bool PRE = false>
__device__ __forceinline__ void epi_qkv(const GemmArgs &a, const float *tile, const float *rstd, int cg, int t,
                                        const float (&pre)[QKV_PRE]) {
    const int tidx = opaque_tid();
    const int hd = a.hd, Hq = a.Hq, Hkv = a.Hkv;
    const int half_hd = hd >> 1;
    const int b = PRE ? __float_as_int(pre[17]) : a.rm.tile_seq[t];
    constexpr int RED_STRIDE = STRIDE;   // the row stride of this tile
    for (int item = tidx; item < 4 * WIDTH; item += 512) {   // GEMM workgroups have 512 threads
        const int row = item & 31, oct = item >> 5;
        const int grow = t * 32 + row;
        const int col0 = cg * WIDTH + oct * 8;     // first of 8 columns, all in one head
        const int kind = col0 < Hq * hd ? 0 : (col0 < (Hq + Hkv) * hd ? 1 : 2);
        const int hc = col0 - (kind == 0 ? 0 : (kind == 1 ? Hq * hd : (Hq + Hkv) * hd));
        const int head = hc / hd, i0 = hc % hd;
        const float sc = rstd[row];
        float v[8];
        if (kind < 2) {
            const int poff = (i0 < half_hd) ? half_hd : -half_hd;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float x = tile[row * RED_STRIDE + oct * 8 + e] * sc;
                float xp = tile[row * RED_STRIDE + oct * 8 + e + poff] * sc;
                const float2 c = PRE ? make_float2(pre[2 * e], pre[2 * e + 1]) : a.cs[(size_t)grow * half_hd + ((i0 + e) % half_hd)];
                v[e] = (i0 < half_hd) ? x * c.x - xp * c.y : x * c.x + xp * c.y;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = tile[row * RED_STRIDE + oct * 8 + e] * sc;
        }
        if (kind == 0) {
            uint4 hi, lo;
            pack8_split(v, hi, lo);
            size_t vec = ((size_t)(t * Hq + head) * (hd / 16)) * 64 + frag_vec(row, i0 >> 3);
            st16<COH>(a.qhi + vec, hi);
            st16<COH>(a.qlo + vec, lo);
        } else {
            const int slot = PRE ? __float_as_int(pre[16]) : a.rm.slot[grow];
            if (slot >= 0) {
                size_t base = (size_t)b * a.kv.seq_stride + (size_t)head * a.kv.head_stride;
                if (kind == 1) {
                    st16<COH>((uint4 *)(a.kv.k + base + k_cache_off(slot, i0 >> 3, hd)), pack8(v));
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        st_u16<COH>(a.kv.vt + base + v_cache_off(slot, i0 + e, hd), (uint16_t)f2bf(v[e]));
                }
            }
        }
    }
}

// The QKV epilogue's own inputs (RoPE factors, cache slot, sequence) of this thread's item, requested before the
// tile is ready so that they are not one more round trip behind it.  One item per thread: WIDTH <= 128.
template <int WIDTH = CG>
__device__ __forceinline__ void qkv_prefetch(const GemmArgs &a, float (&pre)[QKV_PRE], int cg, int t) {
    const int item = opaque_tid();
#pragma unroll
    for (int i = 0; i < QKV_PRE; ++i) pre[i] = 0.f;
    if (item >= 4 * WIDTH) return;
    const int hd = a.hd, Hq = a.Hq, Hkv = a.Hkv, half_hd = hd >> 1;
    const int row = item & 31, oct = item >> 5, grow = t * 32 + row;
    const int col0 = cg * WIDTH + oct * 8;
    const int kind = col0 < Hq * hd ? 0 : (col0 < (Hq + Hkv) * hd ? 1 : 2);
    const int hc = col0 - (kind == 0 ? 0 : (kind == 1 ? Hq * hd : (Hq + Hkv) * hd));
    const int i0 = hc % hd;
    if (kind < 2) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float2 c = a.cs[(size_t)grow * half_hd + ((i0 + e) % half_hd)];
            pre[2 * e] = c.x; pre[2 * e + 1] = c.y;
        }
    }
    if (kind >= 1) pre[16] = __int_as_float(a.rm.slot[grow]);
    pre[17] = __int_as_float(a.rm.tile_seq[t]);
}

// O-proj / down-proj epilogue: h += y; new fragment planes of h; per-group sum of squares.
// `hreg` holds the old h values of this thread's elements e = threadIdx.x + 512*i (row e>>7, column e&127),
// loaded by resid_prefetch() before the tile was ready.  `tile` is overwritten with the new h values.
template <bool COH>
__device__ __forceinline__ void resid_prefetch(const GemmArgs &a, float (&hreg)[8], int cg, int t) {
    const int tidx = opaque_tid();
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int e = tidx + 512 * i;
        const float *hp = a.h + (size_t)(t * 32 + (e >> 7)) * a.N + cg * CG + (e & 127);
        hreg[i] = *hp;
    }
}

template <bool COH>
__device__ __forceinline__ void epi_resid(const GemmArgs &a, float *tile, float *scratch, const float (&hreg)[8], int cg, int t) {
    const int tidx = opaque_tid();
    const int N = a.N;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int e = tidx + 512 * i;
        const int row = e >> 7, col = e & 127;
        const float v = hreg[i] + tile[row * RED_STRIDE + col];
        float *hp = a.h + (size_t)(t * 32 + row) * N + cg * CG + col;
        stf<COH>(hp, v);
        tile[row * RED_STRIDE + col] = v;
    }
    __syncthreads();
    {   // 512 (row, octet) items, one per thread; lanes l and l^32 of a wave hold two octets of the same row
        const int row = tidx & 31, oct = tidx >> 5;
        const float *tp = tile + row * RED_STRIDE + oct * 8;
        uint4 hi, lo;
        pack8_split(tp, hi, lo);
        size_t v = (size_t)t * (N / 16) * 64 + frag_vec(row, cg * 16 + oct);
        st16<COH>(a.xhi_out + v, hi);
        st16<COH>(a.xlo_out + v, lo);
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ss += tp[e] * tp[e];
        ss += shx(ss, 32);
        if ((tidx & 63) < 32) scratch[(tidx >> 6) * 32 + row] = ss;   // [8 waves][32 rows]
    }
    __syncthreads();
    if (a.ssq_sub == 4) {   // wave w holds the octets 2w, 2w + 1: waves 2b, 2b + 1 make 32-column block b
        if (tidx < 128) {
            const int row = tidx & 31, blk = tidx >> 5;
            stf<COH>(a.ssq_out + (size_t)(t * 32 + row) * (N / 32) + cg * 4 + blk,
                     scratch[(2 * blk) * 32 + row] + scratch[(2 * blk + 1) * 32 + row]);
        }
    } else if (tidx < 32) {
        float s2 = 0.f;
#pragma unroll
        for (int w = 0; w < 8; ++w) s2 += scratch[w * 32 + tidx];   // fixed order
        stf<COH>(a.ssq_out + (size_t)(t * 32 + tidx) * (N / CG) + cg, s2);
    }
}

// gate/up epilogue: group = 64 gate + 64 up channels -> SiLU(g) * u, fragment planes over F
template <bool COH>
__device__ __forceinline__ void epi_swiglu(const GemmArgs &a, const float *tile, const float *rstd, int cg, int t) {
    const int tidx = opaque_tid();
    for (int item = tidx; item < 256; item += 512) {
        const int row = item & 31, oct = item >> 5;   // 8 octets of 8 channels
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float g = tile[row * RED_STRIDE + oct * 8 + e] * rstd[row];
            float u = tile[row * RED_STRIDE + 64 + oct * 8 + e] * rstd[row];
            v[e] = g / (1.f + expf(-g)) * u;
        }
        uint4 hi, lo;
        pack8_split(v, hi, lo);
        size_t vec = (size_t)t * (a.F / 16) * 64 + frag_vec(row, cg * 8 + oct);
        st16<COH>(a.ahi + vec, hi);
        st16<COH>(a.alo + vec, lo);
    }
}

// LM-head epilogue: RMSNorm scale, optional logits store, per-(row, group) argmax / sumexp / Gumbel-max.
// LM rows are the first k rows of the tile; lm_row = ct*k + i.
template <bool COH>
__device__ __forceinline__ void epi_lmhead(const GemmArgs &a, const float *tile, const float *rstd, int cg, int ct, int t) {
    const int tidx = opaque_tid();
    if (tidx >= 256) return;
    const int V = a.N, k = a.k;
    const float T = a.T;
    const int row = tidx >> 3, sub = tidx & 7;   // 8 threads per row, 16 columns each
    const bool live = row < k && row >= a.k_lo;
    float m = -INFINITY, gm = -INFINITY, se = 0.f;
    int idx = 0x7fffffff, gidx = 0x7fffffff;
    float z[16];
    const float invT = T > 0.f ? 1.f / T : 1.f;
    if (live) {
        const float sc = rstd[row];
#pragma unroll
        for (int e = 0; e < 16; ++e) z[e] = tile[row * RED_STRIDE + sub * 16 + e] * sc;
        if (a.logits) {
            float *q = a.logits + ((size_t)ct * k + row) * V + (size_t)cg * CG + sub * 16;
#pragma unroll
            for (int e = 0; e < 16; e += 4) *(float4 *)(q + e) = make_float4(z[e], z[e + 1], z[e + 2], z[e + 3]);
        }
        uint64_t key = 0;
        const bool draw = T > 0.f && a.draw;
        if (draw) key = row_key(a.seed, TAG_DRAFT, (uint64_t)a.rm.tile_seq[t], (uint64_t)a.rm.pos[t * 32 + row]);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            int v = cg * CG + sub * 16 + e;
            argmax_merge(m, idx, z[e], v);
            if (draw) argmax_merge(gm, gidx, z[e] * invT + gumbel(key, (uint64_t)v), v);
        }
    }
#pragma unroll
    for (int off = 1; off < 8; off <<= 1) {
        float m2 = shx(m, off); int i2 = shx(idx, off);
        argmax_merge(m, idx, m2, i2);
        float g2 = shx(gm, off); int gi2 = shx(gidx, off);
        argmax_merge(gm, gidx, g2, gi2);
    }
    if (live && T > 0.f) {
#pragma unroll
        for (int e = 0; e < 16; ++e) se += expf((z[e] - m) * invT);
    }
#pragma unroll
    for (int off = 1; off < 8; off <<= 1) se += shx(se, off);
    if (live && sub == 0) {
        RowStat *sp = a.stat + ((size_t)ct * k + row) * a.ncg_v + cg;
        stf<COH>(&sp->m, m); sti<COH>(&sp->idx, idx); stf<COH>(&sp->sumexp, se); stf<COH>(&sp->gm, gm); sti<COH>(&sp->gidx, gidx);
    }
}

// router epilogue: logits over the experts -> softmax -> top_k (lowest index on ties) -> weights
// renormalised to sum 1.  8 threads per row, 16 experts each.
__device__ __forceinline__ void epi_router(const GemmArgs &a, const float *tile, const float *rstd, int t) {
    const int tidx = opaque_tid();
    if (tidx >= 256) return;
    const int row = tidx >> 3, sub = tidx & 7;
    const int grow = t * 32 + row;
    float z[16];
    float m = -INFINITY;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        const int ex = sub * 16 + e;
        z[e] = ex < a.n_experts ? tile[row * RED_STRIDE + ex] * rstd[row] : -INFINITY;
        m = fmaxf(m, z[e]);
    }
#pragma unroll
    for (int off = 1; off < 8; off <<= 1) m = fmaxf(m, shx(m, off));
    float se = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) { z[e] = expf(z[e] - m); se += z[e]; }   // exp(-inf) = 0 for padding
#pragma unroll
    for (int off = 1; off < 8; off <<= 1) se += shx(se, off);
    float wsel[8]; int esel[8];
    float wsum = 0.f;
    for (int j = 0; j < a.top_k; ++j) {
        float bv = -1.f; int bi = 0x7fffffff;
#pragma unroll
        for (int e = 0; e < 16; ++e) argmax_merge(bv, bi, z[e], sub * 16 + e);
#pragma unroll
        for (int off = 1; off < 8; off <<= 1) {
            float v2 = shx(bv, off); int i2 = shx(bi, off);
            argmax_merge(bv, bi, v2, i2);
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) if (sub * 16 + e == bi) z[e] = -1.f;   // taken
        wsel[j] = bv / se; esel[j] = bi;
        wsum += wsel[j];
    }
    if (sub == 0) {
        if (a.route_spread) {
            // benchmarking stand-in for a trained router (a.route_spread - 1 = layer): every row gets top_k distinct
            // pseudo-random experts with equal weights, so a block touches about n (1 - (1 - top_k / n)^rows) experts
            const uint32_t base = (uint32_t)mix64(((uint64_t)a.route_spread << 32) | (uint32_t)grow);
            const uint32_t stride = ((uint32_t)(mix64(base) >> 7) | 1u);   // odd: distinct picks when n is a power of two
            for (int j = 0; j < a.top_k; ++j) {
                a.route_e[grow * 8 + j] = (int)((base + (uint32_t)j * stride) % (uint32_t)a.n_experts);
                a.route_w[grow * 8 + j] = 1.f / (float)a.top_k;
            }
        } else {
            for (int j = 0; j < a.top_k; ++j) {
                a.route_e[grow * 8 + j] = esel[j];
                a.route_w[grow * 8 + j] = wsel[j] / wsum;
            }
        }
    }
}

// RSTD_READY: `rstd` already holds the tile's factors (tile_rstd ran before a barrier the caller has passed).
template <int EPI, bool COH, bool RSTD_READY = false>
__device__ __forceinline__ void run_epilogue(const GemmArgs &a, float *tile, float *rstd, float *scratch,
                                             const float (&hreg)[8], int cg, int ct) {
    // caller has synchronised after filling `tile`
    const int t = a.mt0 + ct * a.mt_stride;
    if (EPI != EPI_RESID && !RSTD_READY) {
        tile_rstd<COH>(a.ssq_in, rstd, t * 32, a.ncg_in, a.d_in, a.eps);
        __syncthreads();
    }
    if (EPI == EPI_QKV) {
        // the wide workgroups load the epilogue's inputs here: requesting them ahead of the tile measured slower
        const float none[QKV_PRE] = {};
        epi_qkv<COH>(a, tile, rstd, cg, t, none);
    }
    else if (EPI == EPI_RESID) epi_resid<COH>(a, tile, scratch, hreg, cg, t);
    else if (EPI == EPI_SWIGLU) epi_swiglu<COH>(a, tile, rstd, cg, t);
    else if (EPI == EPI_ROUTER) epi_router(a, tile, rstd, t);
    else epi_lmhead<COH>(a, tile, rstd, cg, ct, t);
}

// Sum of the 8 waves' accumulators (one 32 x 128 tile each, MFMA register layout) in the fixed order
// w = 0..7, result as a row-major tile (stride RED_STRIDE) in `tile`.
// Every wave parks its 16 register quads in LDS as 16-byte vectors [wave][quad][lane] (conflict-free);
// after one barrier wave w sums quads w and w + 8 over the eight copies (16 independent reads in
// flight per lane) and writes its 8 rows x 64 columns of the tile.  `red` holds 8 * 4096 floats.
// Ends with a barrier.
__device__ __forceinline__ void reduce_waves_to_tile(f32x16 (&acc)[4], float *red, float *tile, int w, int lane) {
    float4 *red4 = (float4 *)red;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            red4[(w * 16 + nb * 4 + q) * 64 + lane] = make_float4(acc[nb][4 * q], acc[nb][4 * q + 1], acc[nb][4 * q + 2], acc[nb][4 * q + 3]);
    barrier_keep_loads();   // LDS traffic only: loads requested earlier (next item, old h) stay in flight
    const int half = lane >> 5, cl = lane & 31;
    float4 v[2][8];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int ww = 0; ww < 8; ++ww) v[j][ww] = red4[(ww * 16 + w + 8 * j) * 64 + lane];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        float4 sum = v[j][0];
#pragma unroll
        for (int ww = 1; ww < 8; ++ww) { sum.x += v[j][ww].x; sum.y += v[j][ww].y; sum.z += v[j][ww].z; sum.w += v[j][ww].w; }
        const int slot = w + 8 * j, nb = slot >> 2, q = slot & 3;
        float *tp = tile + (8 * q + 4 * half) * RED_STRIDE + nb * 32 + cl;   // rows 8q + 4*half + 0..3
        tp[0] = sum.x; tp[RED_STRIDE] = sum.y; tp[2 * RED_STRIDE] = sum.z; tp[3 * RED_STRIDE] = sum.w;
    }
    barrier_keep_loads();   // LDS traffic only: loads requested earlier (next item, old h) stay in flight
}

struct GemmSmem {
    float red[8 * 32 * 128];          // wave-reduction scratch (128 KB)
    float tile[32 * RED_STRIDE];      // the finished 32 x 128 tile, row-major
    float rstd[64];                   // RMSNorm factors of up to two row tiles
    int last;
};

// Sums the S partial tiles of column group cg (row-tile group z) in order s = 0..S-1 and runs the epilogue.
// RSTD_EARLY: sm.rstd already holds the RMSNorm factors of the group's MT row tiles (gemm_block computed them
// while its first weights were on their way).
template <int MT, int EPI, bool COH, bool RSTD_EARLY = false>
__device__ __forceinline__ void gemm_finish(const GemmArgs &a, GemmSmem &sm, int cg, int z) {
    const int tidx = opaque_tid();
    float *tile = sm.tile;
    const int N = a.N, S = a.S;
    float hreg[MT][8];
    float4 v[MT][2];
    // the sums of all MT row tiles first (their loads do not depend on each other's epilogue), then the epilogues
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int ct = z * MT + mt;
        if (EPI == EPI_RESID) resid_prefetch<COH>(a, hreg[mt], cg, a.mt0 + ct * a.mt_stride);
        const size_t sstride = (size_t)a.rows_total * N;
        const float *p[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int e = tidx + 512 * i;
            p[i] = a.part + ((size_t)ct * 32 + (e >> 5)) * N + (size_t)cg * CG + (e & 31) * 4;
            v[mt][i] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
        for (int s0 = 0; s0 < S; s0 += 8) {   // 8 splits x 2 x 16 bytes of loads in flight, summed in order
            u32x4 pv[8][2];
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int i = 0; i < 2; ++i) load16_agent_async(pv[u][i], p[i] + (size_t)min(s0 + u, S - 1) * sstride);
            wait_loads<0>();
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (s0 + u < S) {
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        tie(pv[u][i]);
                        v[mt][i].x += __uint_as_float(pv[u][i][0]); v[mt][i].y += __uint_as_float(pv[u][i][1]);
                        v[mt][i].z += __uint_as_float(pv[u][i][2]); v[mt][i].w += __uint_as_float(pv[u][i][3]);
                    }
                }
        }
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int ct = z * MT + mt;
        if (mt > 0) __syncthreads();
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int e = tidx + 512 * i;
            float *tp = tile + (e >> 5) * RED_STRIDE + (e & 31) * 4;
            tp[0] = v[mt][i].x; tp[1] = v[mt][i].y; tp[2] = v[mt][i].z; tp[3] = v[mt][i].w;
        }
        __syncthreads();
        run_epilogue<EPI, COH, RSTD_EARLY>(a, tile, sm.rstd + 32 * mt, sm.red, hreg[mt], cg, ct);
    }
}

// Debugging aid: thread 0 of workgroup `lin` records the 100 MHz device clock at point i of the launch.
__device__ __forceinline__ void gemm_stamp(const GemmArgs &a, int lin, int i) {
    if (a.stamps && threadIdx.x == 0) a.stamps[lin * 8 + i] = wall_clock64();
}

// One work item of the weight-streaming GEMM: column group cg, K split s, row-tile group z.
// With S > 1 the block that arrives last at the group's counter finishes the group.
// WSTREAM: weights are read once by the whole grid (non-temporal loads); false: several workgroups of an XCD read
// the same weights at about the same time and should find them in its L2 (plain loads).
template <int MT, int EPI, bool COH, bool WSTREAM = true>
__device__ __forceinline__ void gemm_block(const GemmArgs &a, GemmSmem &sm, int cg, int s, int z, int ncg) {
    const int tidx = opaque_tid();
    float *red = sm.red, *tile = sm.tile, *s_rstd = sm.rstd;
    const int w = __builtin_amdgcn_readfirstlane(tidx >> 6), lane = tidx & 63;   // the wave index as a scalar: scalar loop bounds
    const int N = a.N, KS = a.KS, S = a.S;
    // K range of the workgroup: split s of S equal parts; inside it wave w takes the k-steps w, w + 8, w + 16, ...: the
    // eight waves read neighbouring 1 KB fragments at about the same time and advance together (measured against one
    // contiguous eighth per wave: 8B verify pass 4.63 -> 4.60 ms)
    // Splits are whole multiples of 8 k-steps (8 KB per column block): ranges that start anywhere cost 1.4 us per launch
    // of the 8B shape's output projection (7 splits of 36.6 k-steps against 6 of 40 and one of 16).
    constexpr int KSTEP = 8;
    const int per = (KS + S * 8 - 1) / (S * 8);
    const int ks0 = s * 8 * per + w;
    const int ks1 = min(KS, (s + 1) * 8 * per);

    const int lin = (z * S + s) * ncg + cg;   // stamps: 0 start, 1 this wave's K slice multiplied, 2 tile stored
    gemm_stamp(a, lin, 0);                    // (epilogue done if S == 1), 3 arrived, 4 last workgroup's finish done
    f32x16 acc[MT][4];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nb][r] = 0.f;

    const uint4 *wp = a.W + ((size_t)(cg * 4) * KS) * 64 + lane;
    const size_t wstride = (size_t)KS * 64;   // between column blocks
    const uint4 *xh[MT], *xl[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        size_t tl = (size_t)(a.mt0 + (z * MT + mt) * a.mt_stride);
        xh[mt] = a.Xhi + tl * KS * 64 + lane;
        xl[mt] = a.Xlo + tl * KS * 64 + lane;
    }

    // Software pipeline: D k-steps of loads are in flight while older steps are multiplied.  The loads are issued and
    // waited for by hand (load16_async / wait_steps): left to the compiler, the loop waits for ALL outstanding loads once
    // per trip (its count of conditional loads across the back edge is not exact), which empties the pipeline every D
    // k-steps (8B verify pass 4.35 -> 4.26 ms).
    constexpr int D = (MT == 1) ? 4 : 3;   // bounded by the register file: no spills.  (Deeper, 5 or 6 k-steps, or the
    // loads of k-step j + D requested before the products of k-step j through one more buffer: measured, not faster.)
    constexpr int NSLOT = D;
    constexpr int LPS = 4 + 2 * MT;        // loads per k-step
    u32x4 wb[NSLOT][4], xhb[NSLOT][MT], xlb[NSLOT][MT];
    const int n = ks0 < ks1 ? (ks1 - ks0 + KSTEP - 1) / KSTEP : 0;   // this wave's k-steps: ks0, ks0 + 8, ...
    // RMSNorm factors of the input rows: their sums of squares were finished by the previous kernel, so they are
    // requested first and turned into factors once the first k-step has arrived, instead of as a dependent round
    // trip inside the epilogue.  Thread (row, j) = (tidx >> 4, tidx & 15) holds the groups j, j + 16, ...
    constexpr bool RSTD_EARLY = EPI != EPI_RESID;
    constexpr int RSQ = 4;                 // groups per thread: ncg_in <= 64 (the host checks d_model <= 8192)
    float sq[MT][RSQ];
    const int nsq = RSTD_EARLY ? (a.ncg_in + 15) >> 4 : 0;
    if (RSTD_EARLY) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const float *sp = a.ssq_in + (size_t)((a.mt0 + (z * MT + mt) * a.mt_stride) * 32 + (tidx >> 4)) * a.ncg_in;
#pragma unroll
            for (int i = 0; i < RSQ; ++i)
                if (i < nsq) load4_async(sq[mt][i], sp + min((tidx & 15) + 16 * i, a.ncg_in - 1));
        }
    }
    auto request = [&](int sl, int ks) {   // sl is a constant once the callers' loops are unrolled
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) {
            if (WSTREAM) load16_stream_async(wb[sl][nb], wp + nb * wstride + (size_t)ks * 64);
            else load16_async(wb[sl][nb], wp + nb * wstride + (size_t)ks * 64);
        }
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            load16_async(xhb[sl][mt], xh[mt] + (size_t)ks * 64);
            load16_async(xlb[sl][mt], xl[mt] + (size_t)ks * 64);
        }
    };
#pragma unroll
    for (int dd = 0; dd < D; ++dd)
        if (dd < n) request(dd, ks0 + KSTEP * dd);
    for (int j0 = 0; j0 < n; j0 += NSLOT) {
#pragma unroll
        for (int dd = 0; dd < NSLOT; ++dd) {
            const int j = j0 + dd;
            if (j < n) {
                // loads requested after those of k-step j: the k-steps up to j + D - 1
                wait_steps<LPS>(min(D - 1, n - 1 - j));
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) tie(wb[dd][nb]);
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) { tie(xhb[dd][mt]); tie(xlb[dd][mt]); }
                if (RSTD_EARLY && j == 0) {   // the sums of squares were requested before every k-step: they are here
#pragma unroll
                    for (int mt = 0; mt < MT; ++mt) {
                        float ssum = 0.f;
#pragma unroll
                        for (int i = 0; i < RSQ; ++i)
                            if (i < nsq) { tie(sq[mt][i]); if ((tidx & 15) + 16 * i < a.ncg_in) ssum += sq[mt][i]; }
#pragma unroll
                        for (int off = 1; off < 16; off <<= 1) ssum += shx(ssum, off);
                        if ((tidx & 15) == 0) s_rstd[32 * mt + (tidx >> 4)] = rsqrtf(ssum / (float)a.d_in + a.eps);
                    }
                }
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb) {
                        acc[mt][nb] = mfma32(xhb[dd][mt], wb[dd][nb], acc[mt][nb]);
                        acc[mt][nb] = mfma32(xlb[dd][mt], wb[dd][nb], acc[mt][nb]);
                    }
                if (j + D < n) request(dd, ks0 + KSTEP * (j + D));
            }
        }
    }
    if (RSTD_EARLY && n == 0) {   // a wave without k-steps (short K ranges) still owes its rows' factors
        wait_loads<0>();
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            float ssum = 0.f;
#pragma unroll
            for (int i = 0; i < RSQ; ++i)
                if (i < nsq) { tie(sq[mt][i]); if ((tidx & 15) + 16 * i < a.ncg_in) ssum += sq[mt][i]; }
#pragma unroll
            for (int off = 1; off < 16; off <<= 1) ssum += shx(ssum, off);
            if ((tidx & 15) == 0) s_rstd[32 * mt + (tidx >> 4)] = rsqrtf(ssum / (float)a.d_in + a.eps);
        }
    }

    gemm_stamp(a, lin, 1);
    // sum the 8 waves, then either finish (S == 1) or hand the partial tile over
    float hreg[8];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int ct = z * MT + mt;
        if (mt > 0) __syncthreads();
        if (EPI == EPI_RESID && S == 1) resid_prefetch<COH>(a, hreg, cg, a.mt0 + ct * a.mt_stride);
        reduce_waves_to_tile(acc[mt], red, tile, w, lane);
        if (S == 1) {
            run_epilogue<EPI, COH, RSTD_EARLY>(a, tile, s_rstd + 32 * mt, red, hreg, cg, ct);
        } else {
            float *out = a.part + ((size_t)s * a.rows_total + (size_t)ct * 32) * N + (size_t)cg * CG;
#pragma unroll
            for (int i = 0; i < 2; ++i) {   // 16 bytes per lane: a wave writes two rows of the group's 128 columns
                const int e = tidx + 512 * i;
                const int row = e >> 5, c4 = (e & 31) * 4;
                const float *tp = tile + row * RED_STRIDE + c4;
                store16_agent(out + (size_t)row * N + c4, tp[0], tp[1], tp[2], tp[3]);
            }
        }
    }
    gemm_stamp(a, lin, 2);
    if (S == 1) return;
    // the block that arrives last at this column group's counter sums all partials and finishes
    const bool last = arrive_last(a.counters + (size_t)z * ncg + cg, S, &sm.last);
    gemm_stamp(a, lin, 3);
    if (!last) {
        // (sm.red is free: every wave has passed the barrier behind the wave sum)
        if (EPI == EPI_QKV) prefetch_kv(a.kv.k, a.kv.vt, a.kv.head_stride, a.Hkv, a.kv_fetch_bytes, sm.red);
        else prefetch_next(a.nx, sm.red);
        return;
    }
    gemm_finish<MT, EPI, COH, RSTD_EARLY>(a, sm, cg, z);
    gemm_stamp(a, lin, 4);
}

template <int MT, int EPI>
__global__ __launch_bounds__(512) void k_gemm(const GemmArgs a) {
    __shared__ GemmSmem sm;
    gemm_block<MT, EPI, false>(a, sm, blockIdx.x, blockIdx.y, blockIdx.z, gridDim.x);
}

// The same GEMM over Z > 1 row-tile groups (batched passes, prefill chunks): every group needs the same weights.
// 1-D grid; workgroup ids 8 apart run on the same XCD at about the same time, so the Z workgroups of one
// (column group, K split) pair p get the ids 8 * ((p / 8) * Z + z) + p % 8: the first of them to ask for a
// weight line fetches it from memory, the others find it in that XCD's L2.
template <int MT, int EPI>
__global__ __launch_bounds__(512) void k_gemm_rows(const GemmArgs a, int ncg, int Z) {
    __shared__ GemmSmem sm;
    const int lin = blockIdx.x, x = lin & 7, q = lin >> 3;
    const int z = q % Z, p = 8 * (q / Z) + x;
    if (p < ncg * a.S) gemm_block<MT, EPI, false, false>(a, sm, p % ncg, p / ncg, z, ncg);
}

// ------------------------------------------------------------------------------------------
// mixture-of-experts FFN: (row, expert) pairs are grouped per expert, every touched expert's weights
// are streamed once, and the 8 weighted expert outputs of a row are summed in routing order.
// ------------------------------------------------------------------------------------------
// Unsplit GEMMs of a small model in narrow workgroups: NB = 1 (32 columns) for the residual GEMM (O projection),
// NB = 2 (64 columns: whole heads of up to 64 channels) for the QKV projection.
// A 128-column workgroup pulls all of K for four weight blocks and both activation planes through one compute
// unit's L1 (343 KB at K = 896, 64 bytes per clock), and a matrix of 896 columns gives only 7 of them per row
// tile: the launch is bound by those few L1s, then by one SIMD's 112 products and a 128 KB sum through LDS.  Here a
// workgroup owns NB 32-column weight blocks (171 KB through its L1 for one block, 28 products per SIMD, a 32 KB
// sum), and four (two) times as many compute units take part.  Same operand layouts, same order of summation over
// the waves (w = 0..7) and over a wave's k-steps (w, w + 8, ...) as in the wide kernel.
// grid: 1-D, ids 8 apart on one XCD: the Z row tiles of column group p get the ids 8 * ((p / 8) * Z + z) + p % 8.
// Sums of squares are written per 32-column block (GemmArgs::ssq_sub == 4 for every kernel of that model).
// ------------------------------------------------------------------------------------------
template <int NB>
struct GemmNarrowSmem {
    float red[8 * NB * 4 * 64 * 4];   // [wave][register quad][lane][4]
    float tile[32 * (32 * NB + 1)];
    float ssp[2 * 32];
    float rstd[32];
};

template <int NB, int EPI>
__global__ __launch_bounds__(512) void k_gemm_narrow(const GemmArgs a, int ngrp, int Z) {
    static_assert((EPI == EPI_RESID && NB == 1) || (EPI == EPI_QKV && NB == 2), "epilogues exist for these two forms");
    constexpr int TS = 32 * NB + 1;   // row stride of the tile in LDS
    __shared__ GemmNarrowSmem<NB> sm;
    const int lin = blockIdx.x, x8 = lin & 7, q8 = lin >> 3;
    const int z = q8 % Z, p = 8 * (q8 / Z) + x8;
    if (p >= ngrp) return;
    const int tidx = opaque_tid();
    const int w = __builtin_amdgcn_readfirstlane(tidx >> 6), lane = tidx & 63;
    const int N = a.N, KS = a.KS;
    const int t = a.mt0 + z * a.mt_stride;
    const int slin = z * ngrp + p;   // stamps: 0 start, 1 this wave's k-steps multiplied, 2 epilogue done
    gemm_stamp(a, slin, 0);
    const uint4 *wp = a.W + (size_t)(p * NB) * KS * 64 + lane;
    const size_t wstride = (size_t)KS * 64;   // between column blocks
    const uint4 *xh = a.Xhi + (size_t)t * KS * 64 + lane, *xl = a.Xlo + (size_t)t * KS * 64 + lane;
    constexpr int D = NB == 1 ? 8 : 7;   // k-steps of loads in flight per wave (K = 896: all seven of a wave at once)
    uint4 wb[D][NB], xhb[D], xlb[D];
#pragma unroll
    for (int dd = 0; dd < D; ++dd) {
        const int ks = w + 8 * dd;
        if (ks < KS) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) wb[dd][nb] = wp[nb * wstride + (size_t)ks * 64];
            xhb[dd] = xh[(size_t)ks * 64]; xlb[dd] = xl[(size_t)ks * 64];
        }
    }
    float hreg[2];   // RESID: old h of this thread's elements e = tidx + 512 i: row e >> 5, column e & 31
    if (EPI == EPI_RESID) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int e = tidx + 512 * i;
            hreg[i] = a.h[(size_t)(t * 32 + (e >> 5)) * N + p * 32 + (e & 31)];
        }
    } else {   // RMSNorm factors of the input rows, requested behind the first operands
        tile_rstd<false>(a.ssq_in, sm.rstd, t * 32, a.ncg_in, a.d_in, a.eps);
    }
    f32x16 acc[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[nb][r] = 0.f;
    for (int kb = w; kb < KS; kb += 8 * D) {
#pragma unroll
        for (int dd = 0; dd < D; ++dd) {
            const int ks = kb + 8 * dd;
            if (ks < KS) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    acc[nb] = mfma32(xhb[dd], wb[dd][nb], acc[nb]);
                    acc[nb] = mfma32(xlb[dd], wb[dd][nb], acc[nb]);
                }
                const int kn = ks + 8 * D;
                if (kn < KS) {
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) wb[dd][nb] = wp[nb * wstride + (size_t)kn * 64];
                    xhb[dd] = xh[(size_t)kn * 64]; xlb[dd] = xl[(size_t)kn * 64];
                }
            }
        }
    }
    float qpre[QKV_PRE];
    if (EPI == EPI_QKV) qkv_prefetch<32 * NB>(a, qpre, p, t);
    gemm_stamp(a, slin, 1);
    // sum of the 8 waves in the order w = 0..7: wave s < 4 NB sums register quad s & 3 of block s >> 2 and writes
    // its rows 8 q + 4 half + 0..3
    float4 *red4 = (float4 *)sm.red;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int q = 0; q < 4; ++q)
            red4[(w * 4 * NB + nb * 4 + q) * 64 + lane] = make_float4(acc[nb][4 * q], acc[nb][4 * q + 1], acc[nb][4 * q + 2], acc[nb][4 * q + 3]);
    __syncthreads();
    if (w < 4 * NB) {
        float4 sum = red4[w * 64 + lane];
#pragma unroll
        for (int ww = 1; ww < 8; ++ww) {
            const float4 v = red4[(ww * 4 * NB + w) * 64 + lane];
            sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
        }
        float *tp = sm.tile + (8 * (w & 3) + 4 * (lane >> 5)) * TS + (w >> 2) * 32 + (lane & 31);
        tp[0] = sum.x; tp[TS] = sum.y; tp[2 * TS] = sum.z; tp[3 * TS] = sum.w;
    }
    __syncthreads();
    if (EPI == EPI_QKV) {
        epi_qkv<false, 32 * NB, TS, true>(a, sm.tile, sm.rstd, p, t, qpre);
    } else {
        // h += y; new fragment planes of h; sums of squares of the block's 32 columns
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int e = tidx + 512 * i;
            const int row = e >> 5, col = e & 31;
            const float v = hreg[i] + sm.tile[row * TS + col];
            a.h[(size_t)(t * 32 + row) * N + p * 32 + col] = v;
            sm.tile[row * TS + col] = v;
        }
        __syncthreads();
        if (tidx < 128) {   // (row, octet) items: wave 0 has octets 0 and 1, wave 1 octets 2 and 3
            const int row = tidx & 31, oct = tidx >> 5;
            const float *tp = sm.tile + row * TS + oct * 8;
            uint4 hi, lo;
            pack8_split(tp, hi, lo);
            const size_t v = (size_t)t * (N / 16) * 64 + frag_vec(row, p * 4 + oct);
            a.xhi_out[v] = hi;
            a.xlo_out[v] = lo;
            float ss = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += tp[e] * tp[e];
            ss += shx(ss, 32);
            if ((tidx & 63) < 32) sm.ssp[(tidx >> 6) * 32 + row] = ss;
        }
        __syncthreads();
        if (tidx < 32) a.ssq_out[(size_t)(t * 32 + tidx) * (N / 32) + p] = sm.ssp[tidx] + sm.ssp[32 + tidx];
    }
    gemm_stamp(a, slin, 2);
}

// ------------------------------------------------------------------------------------------
// one block: cnt[e], and for pair i of expert e the pass row and its routing slot
__global__ __launch_bounds__(256) void k_moe_group(const int *__restrict__ route_e, const int *__restrict__ row_slot,
                                                   int rows, int top_k, int n_experts, int cap, int *__restrict__ cnt,
                                                   int *__restrict__ pair_row, int *__restrict__ pair_slot,
                                                   unsigned long long *__restrict__ touched_total) {
    __shared__ int s_cnt[128];
    if (threadIdx.x < 128) s_cnt[threadIdx.x] = 0;
    __syncthreads();
    for (int p = threadIdx.x; p < rows * top_k; p += 256) {
        const int row = p / top_k, j = p % top_k;
        if (row_slot[row] < 0) continue;                 // unused rows of a tile route nowhere
        const int e = route_e[row * 8 + j];
        const int i = atomicAdd(&s_cnt[e], 1);           // order inside an expert does not affect results
        pair_row[e * cap + i] = row;
        pair_slot[e * cap + i] = j;
    }
    __syncthreads();
    if (threadIdx.x < n_experts) {
        cnt[threadIdx.x] = s_cnt[threadIdx.x];
        // running count of (layer, expert) pairs whose weights a pass has to stream (for byte accounting)
        if (s_cnt[threadIdx.x] > 0) atomicAdd(touched_total, 1ULL);
    }
}

enum { MOE_GATEUP = 0, MOE_DOWN = 1 };

struct MoeArgs {
    const uint4 *W; size_t wexp_stride;      // expert e's matrix at W + e * wexp_stride (16-byte units)
    const uint4 *Xhi, *Xlo;                  // GATEUP: the pass's fragments of h; DOWN: activation tiles
    int N, KS, cap, chunks;
    const int *cnt, *pair_row, *pair_slot;
    const float *ssq_in; int ncg_in, d_in; float eps;   // GATEUP: RMSNorm scale of each pair's row
    uint4 *ahi, *alo; int Fe;                // GATEUP out: activation tile (e*chunks + chunk), Fe/16 k-steps
    const float *route_w; float *moe_out; int d;        // DOWN out: moe_out[row][slot][d] = w * y
};

#ifndef DEER_MOE_CGS
#define DEER_MOE_CGS 2
#endif
constexpr int MOE_CGS = DEER_MOE_CGS;   // column groups per workgroup of the grouped expert GEMMs
// grid: x = MOE_CGS column groups, y = expert, z = chunk of 32 pairs.  Same streaming loop and wave tree as k_gemm.
// A workgroup does MOE_CGS column groups one after the other and requests the first k-steps of the next before it
// sums and stores the current one: with one workgroup per CU at a time, a launch of many short work items otherwise
// leaves the memory pipe idle during every item's wave sum, epilogue and first-load latency.
template <int MODE>
__global__ __launch_bounds__(512) void k_gemm_moe(const MoeArgs a) {
    __shared__ float red[8 * 32 * 128];
    __shared__ float tile[32 * RED_STRIDE];
    __shared__ float s_rstd[32];
    __shared__ int s_row[32], s_slot[32];
    const int ex = blockIdx.y, chunk = blockIdx.z;
    const int n = a.cnt[ex] - chunk * 32;
    if (n <= 0) return;
    const int ncg = a.N / CG;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, half = lane >> 5, cl = lane & 31;
    const int KS = a.KS;
    if (threadIdx.x < 32) {
        const bool v = threadIdx.x < n;
        s_row[threadIdx.x] = v ? a.pair_row[ex * a.cap + chunk * 32 + threadIdx.x] : -1;
        s_slot[threadIdx.x] = v ? a.pair_slot[ex * a.cap + chunk * 32 + threadIdx.x] : 0;
    }
    __syncthreads();
    if (MODE == MOE_GATEUP && threadIdx.x < 32) {   // RMSNorm factor of each pair's row
        float sc = 0.f;
        const int r = s_row[threadIdx.x];
        if (r >= 0) {
            const float *p = a.ssq_in + (size_t)r * a.ncg_in;
            float ss = 0.f;
            for (int g = 0; g < a.ncg_in; ++g) ss += p[g];
            sc = rsqrtf(ss / (float)a.d_in + a.eps);
        }
        s_rstd[threadIdx.x] = sc;
    }
    const int myrow = s_row[cl];
    const int per = (KS + 7) / 8;
    const int ks0 = w * per, ks1 = min(KS, ks0 + per);
    const size_t wstride = (size_t)KS * 64;
    // activation fragment of this lane: GATEUP gathers the pair's own row out of the pass's tiles
    const uint4 *xh, *xl;
    if (MODE == MOE_GATEUP) {
        const int r = myrow < 0 ? 0 : myrow;
        const size_t off = ((size_t)(r >> 5) * KS) * 64 + (r & 31) + 32 * half;
        xh = a.Xhi + off; xl = a.Xlo + off;
    } else {
        const size_t off = ((size_t)(ex * a.chunks + chunk) * KS) * 64 + lane;
        xh = a.Xhi + off; xl = a.Xlo + off;
    }
    const bool live = myrow >= 0;
    const u32x4 z4 = {0u, 0u, 0u, 0u};
    // D k-steps of loads in flight, issued and waited for by hand (see gemm_block)
    constexpr int D = 4, LPS = 6;
    u32x4 wb[D][4], xhb[D], xlb[D];
    const int nst = max(0, ks1 - ks0);   // this wave's k-steps
    auto request = [&](int sl, const uint4 *wp, int ks) {   // sl is a constant once the callers' loops are unrolled
#pragma unroll
        for (int nb = 0; nb < 4; ++nb) load16_stream_async(wb[sl][nb], wp + nb * wstride + (size_t)ks * 64);
        load16_async(xhb[sl], xh + (size_t)ks * 64);
        load16_async(xlb[sl], xl + (size_t)ks * 64);
    };
    auto first_loads = [&](int cg) {
        const uint4 *wp = a.W + (size_t)ex * a.wexp_stride + ((size_t)(cg * 4) * KS) * 64 + lane;
#pragma unroll
        for (int dd = 0; dd < D; ++dd)
            if (dd < nst) request(dd, wp, ks0 + dd);
    };
    const int cg_first = blockIdx.x * MOE_CGS;
    first_loads(cg_first);
#pragma unroll 1
    for (int it = 0; it < MOE_CGS; ++it) {
        const int cg = cg_first + it;
        if (cg >= ncg) break;
        const uint4 *wp = a.W + (size_t)ex * a.wexp_stride + ((size_t)(cg * 4) * KS) * 64 + lane;
        f32x16 acc[4];
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[nb][r] = 0.f;
        for (int j0 = 0; j0 < nst; j0 += D) {
#pragma unroll
            for (int dd = 0; dd < D; ++dd) {
                const int j = j0 + dd;
                if (j < nst) {
                    wait_steps<LPS>(min(D - 1, nst - 1 - j));   // the k-steps requested after step j
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb) tie(wb[dd][nb]);
                    tie(xhb[dd]); tie(xlb[dd]);
                    const u32x4 ah = live ? xhb[dd] : z4, al = live ? xlb[dd] : z4;
#pragma unroll
                    for (int nb = 0; nb < 4; ++nb) {
                        acc[nb] = mfma32(ah, wb[dd][nb], acc[nb]);
                        acc[nb] = mfma32(al, wb[dd][nb], acc[nb]);
                    }
                    if (j + D < nst) request(dd, wp, ks0 + j + D);
                }
            }
        }
        if (it + 1 < MOE_CGS && cg + 1 < ncg) first_loads(cg + 1);   // on their way during the sum and the epilogue below
        reduce_waves_to_tile(acc, red, tile, w, lane);
        if (MODE == MOE_GATEUP) {
            for (int item = threadIdx.x; item < 256; item += blockDim.x) {
                const int row = item & 31, oct = item >> 5;
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float g = tile[row * RED_STRIDE + oct * 8 + e] * s_rstd[row];
                    float u = tile[row * RED_STRIDE + 64 + oct * 8 + e] * s_rstd[row];
                    v[e] = g / (1.f + expf(-g)) * u;
                }
                uint4 hi, lo;
                pack8_split(v, hi, lo);
                size_t vec = (size_t)(ex * a.chunks + chunk) * (a.Fe / 16) * 64 + frag_vec(row, cg * 8 + oct);
                a.ahi[vec] = hi;
                a.alo[vec] = lo;
            }
        } else {
            for (int e = threadIdx.x; e < 32 * 32; e += blockDim.x) {
                const int row = e >> 5, c4 = (e & 31) * 4;
                const int pr = s_row[row];
                if (pr < 0) continue;
                const int slot = s_slot[row];
                const float wgt = a.route_w[pr * 8 + slot];
                const float *tp = tile + row * RED_STRIDE + c4;
                *(float4 *)(a.moe_out + ((size_t)pr * 8 + slot) * a.d + cg * CG + c4) =
                    make_float4(tp[0] * wgt, tp[1] * wgt, tp[2] * wgt, tp[3] * wgt);
            }
        }
        __syncthreads();   // the tile is read: the next column group's sum may overwrite it
    }
}

// h += sum over the row's experts in routing order; new fragment planes and sums of squares of h
__global__ __launch_bounds__(256) void k_moe_combine(const float *__restrict__ moe_out, const int *__restrict__ row_slot,
                                                     int top_k, float *__restrict__ h, uint4 *__restrict__ xhi,
                                                     uint4 *__restrict__ xlo, float *__restrict__ ssq, int d) {
    __shared__ float tile[32 * RED_STRIDE];
    const int cg = blockIdx.x, t = blockIdx.y, ncg = gridDim.x;
    // 1024 float4 elements of the 32 x 128 tile, four per thread; all loads of a thread are requested before
    // the first is used (the expert outputs of a row are summed in routing order, then added to h)
    float4 hv[4], mv[4][8];
    bool live[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e4 = threadIdx.x + 256 * i, row = e4 >> 5, c4 = (e4 & 31) * 4;
        const int grow = t * 32 + row;
        live[i] = row_slot[grow] >= 0;
        hv[i] = *(const float4 *)(h + (size_t)grow * d + cg * CG + c4);
#pragma unroll
        for (int j = 0; j < 8; ++j)
            mv[i][j] = (live[i] && j < top_k) ? *(const float4 *)(moe_out + ((size_t)grow * 8 + j) * d + cg * CG + c4)
                                              : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e4 = threadIdx.x + 256 * i, row = e4 >> 5, c4 = (e4 & 31) * 4;
        float4 add = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int j = 0; j < 8; ++j) { add.x += mv[i][j].x; add.y += mv[i][j].y; add.z += mv[i][j].z; add.w += mv[i][j].w; }
        float4 v = hv[i];
        if (live[i]) { v.x += add.x; v.y += add.y; v.z += add.z; v.w += add.w; }
        *(float4 *)(h + (size_t)(t * 32 + row) * d + cg * CG + c4) = v;
        float *tp = tile + row * RED_STRIDE + c4;
        tp[0] = v.x; tp[1] = v.y; tp[2] = v.z; tp[3] = v.w;
    }
    __syncthreads();
    tile_to_frag(tile, xhi, xlo, (size_t)t * (d / 16) * 64, cg * CG);
    {   // sum of squares of a row's 128 columns: 8 threads per row, 16 columns each, then a fixed butterfly
        const int row = threadIdx.x >> 3, sub = threadIdx.x & 7;
        float s = 0.f;
#pragma unroll
        for (int c = 0; c < 16; ++c) { const float v = tile[row * RED_STRIDE + sub * 16 + c]; s += v * v; }
#pragma unroll
        for (int off = 1; off < 8; off <<= 1) s += shx(s, off);
        if (sub == 0) ssq[(size_t)(t * 32 + row) * ncg + cg] = s;
    }
}

struct RowResult {   // per LM row
    int argmax;      // lowest index of the max logit
    int sample;      // Gumbel-max sample of softmax(z/T) (T > 0), else = argmax
    float lse;       // log sum exp(z/T) (T > 0), else 0
    float zmax;
};

// one block per LM row: merge the per-group partials
__global__ __launch_bounds__(256) void k_rowstat_final(const RowStat *__restrict__ stat, int ncg_v, float T,
                                                       RowResult *__restrict__ res, int k, int k_lo) {
    __shared__ float sm[256]; __shared__ int si[256]; __shared__ float sg[256]; __shared__ int sgi[256];
    __shared__ float ss[256];
    const int row = blockIdx.x;
    if (row % k < k_lo) return;   // kept from an earlier pass
    const RowStat *p = stat + (size_t)row * ncg_v;
    float m = -INFINITY, gm = -INFINITY; int idx = 0x7fffffff, gidx = 0x7fffffff;
    for (int g = threadIdx.x; g < ncg_v; g += 256) {
        argmax_merge(m, idx, p[g].m, p[g].idx);
        argmax_merge(gm, gidx, p[g].gm, p[g].gidx);
    }
    sm[threadIdx.x] = m; si[threadIdx.x] = idx; sg[threadIdx.x] = gm; sgi[threadIdx.x] = gidx;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (threadIdx.x < off) {
            argmax_merge(sm[threadIdx.x], si[threadIdx.x], sm[threadIdx.x + off], si[threadIdx.x + off]);
            argmax_merge(sg[threadIdx.x], sgi[threadIdx.x], sg[threadIdx.x + off], sgi[threadIdx.x + off]);
        }
        __syncthreads();
    }
    const float M = sm[0];
    float se = 0.f;
    if (T > 0.f) {
        const float invT = 1.f / T;
        for (int g = threadIdx.x; g < ncg_v; g += 256) se += p[g].sumexp * expf((p[g].m - M) * invT);
    }
    ss[threadIdx.x] = se;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (threadIdx.x < off) ss[threadIdx.x] += ss[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        RowResult r;
        const int V = ncg_v * CG;
        r.argmax = (si[0] >= 0 && si[0] < V) ? si[0] : 0;   // a row of NaNs never updates the index
        r.zmax = M;
        if (T > 0.f) { r.sample = (sgi[0] >= 0 && sgi[0] < V) ? sgi[0] : 0; r.lse = M / T + logf(ss[0]); }
        else { r.sample = r.argmax; r.lse = 0.f; }
        res[row] = r;
    }
}

// draft pass tail: draft tokens out, drafter cache length advances over the ingested rows
__global__ void k_draft_finish(SeqState st, const RowResult *__restrict__ res, int *__restrict__ draft, int k, int k_lo) {
    int b = blockIdx.x, i = threadIdx.x;
    if (i < k && i >= k_lo) draft[b * k + i] = res[b * k + i].sample;   // positions below k_lo were fixed by earlier passes
    if (i == 0) { st.dr_len[b] += st.ing_n[b]; st.ing_n[b] = 0; }
}

// ------------------------------------------------------------------------------------------
// block attention for short query blocks over a long GQA cache.
//   Online softmax in fp32.  S^T = K Q^T and O^T = V^T P^T: every MFMA operand is a contraction-contiguous
//   16-byte vector and the softmax row of a lane is its own column.  Key order inside a 32-key tile is
//   permuted (operand row rho holds key 16*((rho/4)%2) + 4*(rho/8) + rho%4) so that a lane's 16 scores are
//   16 consecutive keys.  Q and P enter as (hi, lo) bf16 pairs.
//   With one key range (NS == 1) the result goes straight to the O-projection's input fragments; otherwise
//   each (tile, head, split) leaves an un-normalised partial (M, L, O) in the MFMA register layout and a
//   separate merge combines them (a merge by the last split to finish would serialise NS dependent round
//   trips to memory on one workgroup).
// ------------------------------------------------------------------------------------------
template <int HD>
struct AttnPartial {   // per (tile, head, split): O in register layout [HD/32][8 reg pairs][64 lanes][2], then (M, L)[32]
    static constexpr int O_FLOATS = 32 * HD;
    static constexpr int FLOATS = 32 * HD + 64;
};

template <int HD, bool COH>
__device__ __forceinline__ void attn_write_frag(const f32x16 *o, float inv, int t, int head, int Hq, int lane,
                                                uint4 *__restrict__ xhi, uint4 *__restrict__ xlo, int tt0 = 0,
                                                int ntt = HD / 32) {
    // o[i] holds O^T tile tt0 + i
    // lane (qrow, half) holds dims 32*tt + 8*q + 4*half + 0..3 in regs 4q..4q+3; the partner lane (other
    // half) holds the other 4 dims of the octet.  Half 0 writes octets with even q, half 1 odd q.
    const int half = lane >> 5, qrow = lane & 31;
    const int KS = Hq * HD / 16;
#pragma unroll
    for (int ti = 0; ti < HD / 32; ++ti) {
        if (ti >= ntt) break;
        const int tt = tt0 + ti;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float mine[4], other[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                mine[e] = o[ti][4 * q + e] * inv;
                other[e] = shx(mine[e], 32);
            }
            // octet (tt, q): dims 32*tt + 8*q + 0..7 = half-0 lane's 4 values then half-1 lane's 4 values
            if ((q & 1) == half) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) { v[e] = half ? other[e] : mine[e]; v[4 + e] = half ? mine[e] : other[e]; }
                uint4 hi, lo;
                pack8_split(v, hi, lo);
                size_t vec = (size_t)t * KS * 64 + frag_vec(qrow, head * (HD / 8) + tt * 4 + q);
                st16<COH>(xhi + vec, hi);
                st16<COH>(xlo + vec, lo);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Block attention item for a whole workgroup of 8 waves: passes of many row tiles or long key ranges (k_attn).
//  - one (row tile, kv head, key-range split) item per workgroup; wave w serves query head (w & 3) of the
//    GQA group on the key tiles of parity (w >> 2) of each staged chunk, so two waves per SIMD overlap;
//  - the K and V fragments of a chunk of ATT_CH 32-key tiles are requested by the eight waves together (every
//    fragment fetched once per workgroup instead of once per query head) and land in LDS in fragment order
//    (direct-to-LDS loads, no registers held while they travel); ATT_NBUF chunk buffers form a ring, so
//    ATT_NBUF - 1 chunks are on their way while one is multiplied, with one barrier per chunk;
//  - Q fragments stay in registers, loaded by every wave for its own head;
//  - the two key parities of a head are combined through LDS, then the result goes to the output
//    projection's input (NS == 1) or to an un-normalised partial (M, L, O) for the merge.
// b: the tile's sequence; lim: the key limit of this lane's query row.
// ------------------------------------------------------------------------------------------
#ifndef DEER_ATT_P_LO
#define DEER_ATT_P_LO 1
#endif
constexpr bool ATT_P_LO = DEER_ATT_P_LO != 0;   // the low-order bf16 plane of the softmax weights enters P V
constexpr int ATT_CH = 2;     // key tiles per staged chunk: one per key parity
constexpr int ATT_NBUF = 4;   // chunk buffers: ATT_NBUF - 1 chunks (96 KB) are on their way while one is multiplied
struct AttnSmem {
    uint4 buf[ATT_NBUF][ATT_CH * 16 * 64];   // [tile][fragment: K k-steps, then V (tile, half) pairs][lane]; 4 x 32 KB
    float2 ml[4 * 64];                       // parked (m, l) of the odd-parity waves
};

// FRAGS_EARLY: all K fragments of a tile are requested from LDS before the first product and the V fragments
// before the softmax, so the matrix pipe does not wait for one LDS read per two products.
template <int HD, bool FRAGS_EARLY = false>
__device__ __forceinline__ void attn_item(const uint4 *Qhi, const uint4 *Qlo, const uint16_t *__restrict__ Kc,
                                          const uint16_t *__restrict__ Vt, size_t seq_stride, size_t head_stride,
                                          int max_seq, int b, int lim, float *part, int Hq, int Hkv, int NS,
                                          float scale_log2e, uint4 *xhi, uint4 *xlo, AttnSmem &as, int kvh, int split, int t) {
    constexpr int KSQ = HD / 16, HT = HD / 32, FPT = KSQ + 2 * HT;   // fragments per tile
    constexpr int LPW = ATT_CH * FPT / 8;                            // staging loads per wave and chunk
    constexpr int PF = AttnPartial<HD>::FLOATS;
    const int tidx = opaque_tid();
    const int w = __builtin_amdgcn_readfirstlane(tidx >> 6), lane = tidx & 63;   // the wave index as a scalar
    const int G = Hq / opaque_s(Hkv);
    // up to four query heads per kv head: wave = (head, key-tile parity); more: wave = head, every key tile, so
    // that eight heads share one pass over the keys instead of two
    const bool wide = G > 4;
    const int g = wide ? w : (w & 3), par = wide ? 0 : (w >> 2);
    const int npar = wide ? 1 : 2, hpr = wide ? 8 : 4;   // key parities; heads per round
    const int half = lane >> 5, qrow = lane & 31;
    int maxlim = lim, minlim = lim;
#pragma unroll
    for (int off = 1; off < 32; off <<= 1) {
        maxlim = max(maxlim, shx(maxlim, off));
        minlim = min(minlim, shx(minlim, off));
    }
    const int nkt = (maxlim + 31) >> 5;
    const int per = (nkt + NS - 1) / opaque_s(NS);
    const int kt0 = split * per, kt1 = min(nkt, kt0 + per);
    const int nchunks = kt1 > kt0 ? (kt1 - kt0 + ATT_CH - 1) / ATT_CH : 0;
    const uint16_t *Kp = Kc + (size_t)b * seq_stride + (size_t)kvh * head_stride;
    const uint16_t *Vp = Vt + (size_t)b * seq_stride + (size_t)kvh * head_stride;

    // Requests this wave's share of a chunk (fragment f = w + 8 * i) straight into LDS: a 16-byte
    // direct-to-LDS load writes lane l's vector at (uniform base) + 16 * l, which is the fragment order, and
    // needs no registers while it travels.  Tiles past the range repeat the last one (not used).
    auto stage = [&](uint4 *dst, int c0) {
        const int ntile = min(ATT_CH, kt1 - c0);
        // the lane offset (elements) is rebuilt here from a small value, so that 64-bit addresses per lane do not
        // live (spilled) across the whole item
        int lo8 = lane * 8;
        asm volatile("" : "+v"(lo8));
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int f = w + 8 * i, tl = f / FPT, fi = f % FPT;
            const int kt = c0 + min(tl, ntile - 1);
            const uint16_t *src;   // both caches hold a key tile as HD / 16 fragments of 1 KB
            if (fi < KSQ) src = Kp + (lo8 + kt * (32 * HD) + fi * 512);
            else src = Vp + (lo8 + kt * (32 * HD) + (fi - KSQ) * 512);
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)src,
                                             (void __attribute__((address_space(3))) *)(dst + f * 64), 16, 0, 0);
        }
    };

    for (int g0 = 0; g0 < G; g0 += hpr) {
        const bool active = g0 + g < G;
        const int head = kvh * G + min(g0 + g, G - 1);
        f32x16 oacc[HT];
#pragma unroll
        for (int tt = 0; tt < HT; ++tt)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[tt][r] = 0.f;
        float m_run = -INFINITY, l_run = 0.f;

        if (nchunks > 0) {
            uint4 qh[KSQ], ql[KSQ];
            __syncthreads();   // the previous head round or item has been read
            {   // this wave's Q fragments (requested first: every later wait covers them)
                const size_t qb = ((size_t)(t * Hq + head) * KSQ) * 64 + lane;
#pragma unroll
                for (int s = 0; s < KSQ; ++s) { qh[s] = Qhi[qb + (size_t)s * 64]; ql[s] = Qlo[qb + (size_t)s * 64]; }
            }
#pragma unroll
            for (int c = 0; c < ATT_NBUF - 1; ++c)
                if (c < nchunks) stage(as.buf[c], kt0 + c * ATT_CH);

            for (int ci = 0; ci < nchunks; ++ci) {
                const int c0 = kt0 + ci * ATT_CH;
                const int ntile = min(ATT_CH, kt1 - c0);
                // chunk ci has landed once at most the loads of the chunks requested after it are outstanding
                const int later = min(ATT_NBUF - 2, nchunks - 1 - ci);
                if (later >= 2) wait_loads<2 * LPW>(); else if (later == 1) wait_loads<LPW>(); else wait_loads<0>();
                barrier_keep_loads();   // every wave's share of chunk ci is in LDS, and chunk ci - 1 has been read by all
                if (ci + ATT_NBUF - 1 < nchunks) stage(as.buf[(ci + ATT_NBUF - 1) % ATT_NBUF], c0 + (ATT_NBUF - 1) * ATT_CH);
                if (active)
                for (int tl = par; tl < ntile; tl += npar) {
                    const int kt = c0 + tl;
                    const uint4 *fr = as.buf[ci % ATT_NBUF] + (size_t)(tl * FPT) * 64 + lane;
                    f32x16 sacc;
#pragma unroll
                    for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
                    uint4 kf[KSQ], vfr[HT * 2];
                    if (FRAGS_EARLY) {
#pragma unroll
                        for (int s = 0; s < KSQ; ++s) kf[s] = fr[s * 64];
                        __builtin_amdgcn_sched_barrier(0);
                    }
#pragma unroll
                    for (int s = 0; s < KSQ; ++s) {
                        if (!FRAGS_EARLY) kf[s] = fr[s * 64];
                        sacc = mfma32(kf[s], qh[s], sacc);
                        sacc = mfma32(kf[s], ql[s], sacc);
                    }
                    if (FRAGS_EARLY) {
#pragma unroll
                        for (int i = 0; i < HT * 2; ++i) vfr[i] = fr[(KSQ + i) * 64];
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    // lane holds keys kt*32 + 16*half + r, r = 0..15, for query row qrow
                    const int key0 = kt * 32 + 16 * half;
                    if (kt * 32 + 32 > minlim) {   // only tiles that reach some row's limit need the mask
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (key0 + r >= lim) sacc[r] = -INFINITY;
                    }
                    float mx = sacc[0];
#pragma unroll
                    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sacc[r]);
                    mx = fmaxf(mx, shx(mx, 32));
                    const float m_new = fmaxf(m_run, mx);
                    float pr[16];
                    if (m_new == -INFINITY) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) pr[r] = 0.f;
                    } else {
                        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2e);   // m_run = -inf -> 0
                        const float mb = m_new * scale_log2e;
                        float ls = 0.f;
#pragma unroll
                        for (int r = 0; r < 16; ++r) { pr[r] = __builtin_amdgcn_exp2f(sacc[r] * scale_log2e - mb); ls += pr[r]; }
                        l_run = l_run * alpha + ls;
                        m_run = m_new;
                        if (__builtin_amdgcn_ballot_w64(alpha != 1.f)) {   // the running max moved for some row
#pragma unroll
                            for (int tt = 0; tt < HT; ++tt)
#pragma unroll
                                for (int r = 0; r < 16; ++r) oacc[tt][r] *= alpha;
                        }
                    }
                    uint4 ph[2], pl[2];
                    pack8_split(pr, ph[0], pl[0]);
                    pack8_split(pr + 8, ph[1], pl[1]);
#pragma unroll
                    for (int tt = 0; tt < HT; ++tt)
#pragma unroll
                        for (int s2 = 0; s2 < 2; ++s2) {
                            const uint4 vf = FRAGS_EARLY ? vfr[tt * 2 + s2] : fr[(KSQ + tt * 2 + s2) * 64];
                            oacc[tt] = mfma32(vf, ph[s2], oacc[tt]);
                            if (ATT_P_LO) oacc[tt] = mfma32(vf, pl[s2], oacc[tt]);
                        }
                }
            }
            __syncthreads();   // the buffers have been read: the parity merge below reuses them
        } else {
            __syncthreads();   // the previous head round or item has been read
        }
        // combine the two key parities of each head: odd-parity waves park (m, l, O), even-parity waves merge
        float4 *ox = (float4 *)as.buf[0];
        if (par == 1) {   // never in the one-wave-per-head arrangement
            as.ml[g * 64 + lane] = make_float2(m_run, l_run);
#pragma unroll
            for (int tt = 0; tt < HT; ++tt)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    ox[((g * HT + tt) * 4 + q) * 64 + lane] = make_float4(oacc[tt][4 * q], oacc[tt][4 * q + 1], oacc[tt][4 * q + 2], oacc[tt][4 * q + 3]);
        }
        __syncthreads();
        if (par == 0 && active) {
            if (!wide) {
                const float2 o_ml = as.ml[g * 64 + lane];
                const float M = fmaxf(m_run, o_ml.x);
                const float f0 = (m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((m_run - M) * scale_log2e);
                const float f1 = (o_ml.x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((o_ml.x - M) * scale_log2e);
                l_run = f0 * l_run + f1 * o_ml.y;
                m_run = M;
#pragma unroll
                for (int tt = 0; tt < HT; ++tt)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float4 v = ox[((g * HT + tt) * 4 + q) * 64 + lane];
                        oacc[tt][4 * q] = f0 * oacc[tt][4 * q] + f1 * v.x;
                        oacc[tt][4 * q + 1] = f0 * oacc[tt][4 * q + 1] + f1 * v.y;
                        oacc[tt][4 * q + 2] = f0 * oacc[tt][4 * q + 2] + f1 * v.z;
                        oacc[tt][4 * q + 3] = f0 * oacc[tt][4 * q + 3] + f1 * v.w;
                    }
            }
            const float l_tot = l_run + shx(l_run, 32);
            if (NS == 1) {
                attn_write_frag<HD, true>(oacc, l_tot > 0.f ? 1.f / l_tot : 0.f, t, head, Hq, lane, xhi, xlo);
            } else {
                float *pp = part + ((size_t)(t * Hq + head) * NS + split) * PF;
#pragma unroll
                for (int tt = 0; tt < HT; ++tt)
#pragma unroll
                    for (int r2 = 0; r2 < 8; ++r2) st_agent2(pp + ((tt * 8 + r2) * 64 + lane) * 2, oacc[tt][2 * r2], oacc[tt][2 * r2 + 1]);
                if (half == 0) st_agent2(pp + 32 * HD + 2 * qrow, m_run, l_tot);
            }
        }
    }
}

// grid: x = kv_head + Hkv * split, y = pass tile (32 query rows of one sequence); 512 threads
template <int HD>
__global__ __launch_bounds__(512) void k_attn(const uint4 *__restrict__ Qhi, const uint4 *__restrict__ Qlo,
                                              const uint16_t *__restrict__ Kc, const uint16_t *__restrict__ Vt,
                                              size_t seq_stride, size_t head_stride, int max_seq,
                                              const int *__restrict__ tile_seq, const int *__restrict__ row_limit,
                                              float *__restrict__ part, int Hq, int Hkv, int NS, float scale_log2e,
                                              uint4 *__restrict__ xhi, uint4 *__restrict__ xlo) {
    __shared__ __attribute__((aligned(16))) AttnSmem as;
    const int t = blockIdx.y;
    attn_item<HD, true>(Qhi, Qlo, Kc, Vt, seq_stride, head_stride, max_seq, tile_seq[t], row_limit[t * 32 + (threadIdx.x & 31)],
                        part, Hq, Hkv, NS, scale_log2e, xhi, xlo, as, blockIdx.x % Hkv, blockIdx.x / Hkv, t);
}

// Writes registers 8*hh .. 8*hh+7 of O^T tile tt (held in o[0..7], scaled by inv) into the output projection's
// input fragments: octets q = 2*hh and 2*hh + 1 (see attn_write_frag for the lane pairing).
template <int HD>
__device__ __forceinline__ void attn_store_slice(const float (&o)[8], float inv, int Hq, int head, int t, int tt, int hh,
                                                 int lane, uint4 *xhi, uint4 *xlo) {
    const int half = lane >> 5, qrow = lane & 31;
    const int KS = Hq * HD / 16;
#pragma unroll
    for (int qq = 0; qq < 2; ++qq) {
        const int q = 2 * hh + qq;
        float mine[4], other[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) { mine[e] = o[4 * qq + e] * inv; other[e] = shx(mine[e], 32); }
        if ((q & 1) == half) {
            float v8[8];
#pragma unroll
            for (int e = 0; e < 4; ++e) { v8[e] = half ? other[e] : mine[e]; v8[4 + e] = half ? mine[e] : other[e]; }
            uint4 hi, lo;
            pack8_split(v8, hi, lo);
            const size_t vec = (size_t)t * KS * 64 + frag_vec(qrow, head * (HD / 8) + tt * 4 + q);
            st16<true>(xhi + vec, hi);
            st16<true>(xlo + vec, lo);
        }
    }
}

// Merge of the NS key-range partials of one (tile, head): wave item (tt, hh) owns register pairs 4*hh .. 4*hh+3
// of O^T tile tt.  All (M, L) pairs are requested at once, then the partial outputs 16 splits at a time, so a
// merge of 32 splits is three memory round trips.  Splits are combined in order s = 0..NS-1.  NS <= 32.
// EARLY (the merge kernel, which has the registers for it): the first 16 partial outputs are requested together
// with the (M, L) pairs, which makes it two round trips.
template <int HD, bool EARLY = false>
__device__ __forceinline__ void attn_merge_item(const float *part, int NS, int Hq, float scale_log2e, uint4 *xhi, uint4 *xlo,
                                                int head, int t, int tt, int hh, int lane) {
    constexpr int PF = AttnPartial<HD>::FLOATS;
    const int half = lane >> 5, qrow = lane & 31;
    const float *p0 = part + (size_t)(t * Hq + head) * NS * PF;
    float f[32];
    float M = -INFINITY, L = 0.f;
    float2 v[16][4];
    auto load_half = [&](int s0) {
#pragma unroll
        for (int u = 0; u < 16; ++u)
#pragma unroll
            for (int r2 = 0; r2 < 4; ++r2)
                v[u][r2] = ld_agent2(p0 + (size_t)min(s0 + u, NS - 1) * PF + ((tt * 8 + 4 * hh + r2) * 64 + lane) * 2);
    };
    if (EARLY) load_half(0);
    {
        float2 ml[32];
#pragma unroll
        for (int s = 0; s < 32; ++s) ml[s] = ld_agent2(p0 + (size_t)min(s, NS - 1) * PF + 32 * HD + 2 * qrow);
#pragma unroll
        for (int s = 0; s < 32; ++s) if (s < NS) M = fmaxf(M, ml[s].x);
#pragma unroll
        for (int s = 0; s < 32; ++s) {
            f[s] = (s >= NS || ml[s].x == -INFINITY) ? 0.f : exp2f((ml[s].x - M) * scale_log2e);
            L += f[s] * ml[s].y;
        }
    }
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.f;
#pragma unroll
    for (int s0 = 0; s0 < 32; s0 += 16) {
        if (s0 < NS) {
            if (!(EARLY && s0 == 0)) load_half(s0);
#pragma unroll
            for (int u = 0; u < 16; ++u)
#pragma unroll
                for (int r2 = 0; r2 < 4; ++r2) { o[2 * r2] += f[s0 + u] * v[u][r2].x; o[2 * r2 + 1] += f[s0 + u] * v[u][r2].y; }
        }
    }
    attn_store_slice<HD>(o, L > 0.f ? 1.f / L : 0.f, Hq, head, t, tt, hh, lane, xhi, xlo);
}

// grid: one wave per (tile, head, O^T tile, half): 256 threads = 4 wave items per block
template <int HD>
__global__ __launch_bounds__(256) void k_attn_merge(const float *__restrict__ part, int NS, int Hq, int n_items,
                                                    float scale_log2e, uint4 *__restrict__ xhi, uint4 *__restrict__ xlo) {
    constexpr int HT = HD / 32;
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= n_items) return;
    const int hh = j & 1, tt = (j >> 1) % HT, head = (j / (2 * HT)) % Hq, t = j / (2 * HT * Hq);
    attn_merge_item<HD, true>(part, NS, Hq, scale_log2e, xhi, xlo, head, t, tt, hh, threadIdx.x & 63);
}

// Merge of the NS key-range partials of one (tile, head) written by attn_head_item: wave item (tt, hh) owns registers
// 8*hh .. 8*hh+7 of O^T tile tt, which a partial holds as two register quads of 1 KB per wave.  All (M, L) pairs and the
// outputs of the first 8 ranges (16 with head_dim <= 64) are requested together: one round trip for that many ranges;
// ranges are combined in order s = 0..NS-1.  NS <= 32.
template <int HD>
__device__ __forceinline__ void attn_head_merge(const float *part, int NS, int Hq, float scale_log2e, uint4 *xhi, uint4 *xlo,
                                                int head, int t, int tt, int hh, int lane) {
    constexpr int PF = AttnPartial<HD>::FLOATS;
    const int qrow = lane & 31;
    const float *p0 = part + (size_t)(t * Hq + head) * NS * PF;
    const float *po = p0 + ((tt * 2 + hh) * 2 * 64 + lane) * 4;
    constexpr int CH = HD <= 64 ? 16 : 8;   // ranges whose outputs are requested together (registers: 8 per range)
    u32x4 v[CH][2];
    auto request = [&](int s0) {
#pragma unroll
        for (int u = 0; u < CH; ++u)
            if (s0 + u < NS) {
                load16_agent_async(v[u][0], po + (size_t)(s0 + u) * PF);
                load16_agent_async(v[u][1], po + (size_t)(s0 + u) * PF + 256);
            }
    };
    float f[32];
    float M = -INFINITY, L = 0.f;
    {
        float2 ml[32];
#pragma unroll
        for (int s = 0; s < 32; ++s) ml[s] = ld_agent2(p0 + (size_t)min(s, NS - 1) * PF + 32 * HD + 2 * qrow);
        request(0);
#pragma unroll
        for (int s = 0; s < 32; ++s) if (s < NS) M = fmaxf(M, ml[s].x);
#pragma unroll
        for (int s = 0; s < 32; ++s) {
            f[s] = (s >= NS || ml[s].x == -INFINITY) ? 0.f : exp2f((ml[s].x - M) * scale_log2e);
            L += f[s] * ml[s].y;
        }
    }
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.f;
#pragma unroll
    for (int s0 = 0; s0 < 32; s0 += CH) {
        if (s0 < NS) {
            if (s0 > 0) request(s0);
            wait_loads<0>();
#pragma unroll
            for (int u = 0; u < CH; ++u)
                if (s0 + u < NS) {
                    tie(v[u][0]); tie(v[u][1]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        o[e] += f[s0 + u] * __uint_as_float(v[u][0][e]);
                        o[4 + e] += f[s0 + u] * __uint_as_float(v[u][1][e]);
                    }
                }
        }
    }
    attn_store_slice<HD>(o, L > 0.f ? 1.f / L : 0.f, Hq, head, t, tt, hh, lane, xhi, xlo);
}

// ------------------------------------------------------------------------------------------
// Block attention for passes of few row tiles (decoding: draft and verify passes of small batches), one
// (row tile, query head, key range) item per workgroup.  Against k_attn + k_attn_merge this spreads a pass of
// one tile over every compute unit with 8 key ranges instead of 32, so the partial results are a quarter as
// large, and needs no second kernel: the last workgroup of a head to arrive merges the ranges itself.
//  - All eight waves serve the same head; wave w takes the key tiles w, w + 8, ... of the range and keeps
//    its own running (m, l, O).  No barrier inside the key loop: a wave's tiles are its own.
//  - A wave has two key tiles on their way at any time: one lands in its private LDS slot (direct-to-LDS
//    loads, no registers while they travel), the next one in registers; tiles alternate between the two.
//  - Q (hi and lo planes of the head) is staged once in LDS and shared by the waves.
//  - The eight running states are combined through LDS (every wave parks its O in its own slot, then wave
//    (tt, hh) sums register group hh of O^T tile tt over the eight copies in wave order); with one key range
//    the result is final, otherwise it is this range's partial and the ranges meet at an arrival counter.
// The kv heads of the K/V cache are shared by the G query heads of a group through the L2 of their XCD:
// workgroup ids cycle through the kv heads first, so with 8 kv heads every XCD serves one of them.
// ------------------------------------------------------------------------------------------
template <int HD>
struct AttnHeadSmem {
    uint4 slot[8][(HD / 8) * 64];   // per wave: one key tile (K k-step fragments, then V^T fragments); later its parked O
    uint4 q[(HD / 8) * 64];         // Q fragments of the head: hi plane, then lo plane
    float2 ml[8 * 64];              // parked (m, l) per wave and lane
    int last;
};

template <int HD>
__device__ __forceinline__ void attn_head_item(const uint4 *Qhi, const uint4 *Qlo, const uint16_t *__restrict__ Kc,
                                               const uint16_t *__restrict__ Vt, size_t seq_stride, size_t head_stride,
                                               int b, int lim, float *part, int *counters, int Hq, int Hkv, int NS,
                                               float scale_log2e, uint4 *xhi, uint4 *xlo, AttnHeadSmem<HD> &as, int head,
                                               int split, int t, const NextWeights &nx) {
    constexpr int HT = HD / 32, KSQ = HD / 16, FPT = KSQ + 2 * HT;   // fragments (1 KB each) per key tile
    constexpr int PF = AttnPartial<HD>::FLOATS;
    const int tidx = opaque_tid();
    const int w = __builtin_amdgcn_readfirstlane(tidx >> 6), lane = tidx & 63;
    const int half = lane >> 5, qrow = lane & 31;
    int maxlim = lim, minlim = lim;
#pragma unroll
    for (int off = 1; off < 32; off <<= 1) {
        maxlim = max(maxlim, shx(maxlim, off));
        minlim = min(minlim, shx(minlim, off));
    }
    maxlim = __builtin_amdgcn_readfirstlane(maxlim);
    minlim = __builtin_amdgcn_readfirstlane(minlim);
    const int nkt = (maxlim + 31) >> 5;
    const int per = (nkt + NS - 1) / opaque_s(NS);
    const int kt0 = split * per, kt1 = min(nkt, kt0 + per);
    const int first = kt0 + w;                                  // this wave's tiles: first, first + 8, ...
    const int n = first < kt1 ? (kt1 - first + 7) >> 3 : 0;
    const int kvh = head / (Hq / opaque_s(Hkv));
    const uint16_t *Kp = Kc + (size_t)b * seq_stride + (size_t)kvh * head_stride;
    const uint16_t *Vp = Vt + (size_t)b * seq_stride + (size_t)kvh * head_stride;
    uint4 *myslot = as.slot[w];

    // fragment f of key tile kt as this lane reads it: K k-step f, or V^T (O^T tile, key half) pair f - KSQ
    auto frag_src = [&](int kt, int f) -> const uint16_t * {   // both caches hold a key tile as HD / 16 fragments of 1 KB
        int lo8 = lane * 8;
        asm volatile("" : "+v"(lo8));
        if (f < KSQ) return Kp + (lo8 + kt * (32 * HD) + f * 512);
        return Vp + (lo8 + kt * (32 * HD) + (f - KSQ) * 512);
    };
    auto issue_lds = [&](int kt) {
#pragma unroll
        for (int f = 0; f < FPT; ++f)
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)frag_src(kt, f),
                                             (void __attribute__((address_space(3))) *)(myslot + f * 64), 16, 0, 0);
    };
    u32x4 rf[FPT];   // the key tile that travels in registers
    auto issue_reg = [&](int kt) {
#pragma unroll
        for (int f = 0; f < FPT; ++f) load16_async(rf[f], frag_src(kt, f));
    };

    // Q first (every later wait covers it), then this wave's first two key tiles
    {
        const size_t qb = ((size_t)(t * Hq + head) * KSQ) * 64 + lane;
        for (int f = w; f < 2 * KSQ; f += 8) {
            const uint4 *src = f < KSQ ? Qhi + qb + (size_t)f * 64 : Qlo + qb + (size_t)(f - KSQ) * 64;
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1))) *)src,
                                             (void __attribute__((address_space(3))) *)(as.q + f * 64), 16, 0, 0);
        }
    }
    if (n > 0) issue_lds(first);
    if (n > 1) issue_reg(first + 8);
    if (n > 1) wait_loads<2 * FPT>(); else if (n == 1) wait_loads<FPT>(); else wait_loads<0>();
    barrier_keep_loads();   // Q of every wave's share is in LDS

    f32x16 oacc[HT];
#pragma unroll
    for (int tt = 0; tt < HT; ++tt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[tt][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const uint4 *qf = as.q + lane;

    // one key tile: S^T = K Q^T, running softmax, O^T += V^T P^T; FROM_LDS: fragments from the slot, else from rf
    auto tile = [&](auto from_lds, int kt) {
        constexpr bool FROM_LDS = decltype(from_lds)::value;
        const uint4 *fr = myslot + lane;
        f32x16 sacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
        for (int s = 0; s < KSQ; ++s) {
            const uint4 qh = qf[s * 64], ql = qf[(KSQ + s) * 64];
            if (FROM_LDS) {
                const uint4 kf = fr[s * 64];
                sacc = mfma32(kf, qh, sacc);
                sacc = mfma32(kf, ql, sacc);
            } else {
                sacc = mfma32(rf[s], qh, sacc);
                sacc = mfma32(rf[s], ql, sacc);
            }
        }
        const int key0 = kt * 32 + 16 * half;   // lane holds keys key0 + r, r = 0..15, for query row qrow
        if (kt * 32 + 32 > minlim) {            // only tiles that reach some row's limit need the mask
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (key0 + r >= lim) sacc[r] = -INFINITY;
        }
        float mx = sacc[0];
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, sacc[r]);
        mx = fmaxf(mx, shx(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        float pr[16];
        if (m_new == -INFINITY) {
#pragma unroll
            for (int r = 0; r < 16; ++r) pr[r] = 0.f;
        } else {
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2e);   // m_run = -inf -> 0
            const float mb = m_new * scale_log2e;
            float ls = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) { pr[r] = __builtin_amdgcn_exp2f(sacc[r] * scale_log2e - mb); ls += pr[r]; }
            l_run = l_run * alpha + ls;
            m_run = m_new;
            if (__builtin_amdgcn_ballot_w64(alpha != 1.f)) {   // the running max moved for some row
#pragma unroll
                for (int tt = 0; tt < HT; ++tt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[tt][r] *= alpha;
            }
        }
        uint4 ph[2], pl[2];
        pack8_split(pr, ph[0], pl[0]);
        pack8_split(pr + 8, ph[1], pl[1]);
#pragma unroll
        for (int tt = 0; tt < HT; ++tt)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                if (FROM_LDS) {
                    const uint4 vf = fr[(KSQ + tt * 2 + s2) * 64];
                    oacc[tt] = mfma32(vf, ph[s2], oacc[tt]);
                    if (ATT_P_LO) oacc[tt] = mfma32(vf, pl[s2], oacc[tt]);
                } else {
                    oacc[tt] = mfma32(rf[KSQ + tt * 2 + s2], ph[s2], oacc[tt]);
                    if (ATT_P_LO) oacc[tt] = mfma32(rf[KSQ + tt * 2 + s2], pl[s2], oacc[tt]);
                }
            }
    };

    // loads return in order: Q, tile 0 (LDS), tile 1 (registers), tile 2 (LDS, requested after tile 0 was used), ...
    for (int i = 0; i < n; i += 2) {
        if (i + 1 < n) wait_loads<FPT>(); else wait_loads<0>();
        tile(std::true_type{}, first + 8 * i);
        if (i + 2 < n) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the slot has been read
            issue_lds(first + 8 * (i + 2));
        }
        if (i + 1 < n) {
            if (i + 2 < n) wait_loads<FPT>(); else wait_loads<0>();
#pragma unroll
            for (int f = 0; f < FPT; ++f) tie(rf[f]);
            tile(std::false_type{}, first + 8 * (i + 1));
            if (i + 3 < n) issue_reg(first + 8 * (i + 3));
        }
    }

    // park (m, l) and O; the slot is this wave's own, its loads have landed and its reads are done
    const float l_tot = l_run + shx(l_run, 32);
    as.ml[w * 64 + lane] = make_float2(m_run, l_tot);
    {
        float4 *ox = (float4 *)myslot;
#pragma unroll
        for (int tt = 0; tt < HT; ++tt)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                ox[(tt * 4 + q) * 64 + lane] = make_float4(oacc[tt][4 * q], oacc[tt][4 * q + 1], oacc[tt][4 * q + 2], oacc[tt][4 * q + 3]);
    }
    __syncthreads();
    if (w < 2 * HT) {   // wave (tt, hh): registers 8*hh .. 8*hh+7 of O^T tile tt, summed over the waves in order
        const int tt = w >> 1, hh = w & 1;
        float2 ml[8];
        float M = -INFINITY, L = 0.f, f[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) { ml[u] = as.ml[u * 64 + lane]; M = fmaxf(M, ml[u].x); }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            f[u] = (ml[u].x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((ml[u].x - M) * scale_log2e);
            L += f[u] * ml[u].y;
        }
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float4 *ox = (const float4 *)as.slot[u];
            const float4 a0 = ox[(tt * 4 + 2 * hh) * 64 + lane], a1 = ox[(tt * 4 + 2 * hh + 1) * 64 + lane];
            o[0] += f[u] * a0.x; o[1] += f[u] * a0.y; o[2] += f[u] * a0.z; o[3] += f[u] * a0.w;
            o[4] += f[u] * a1.x; o[5] += f[u] * a1.y; o[6] += f[u] * a1.z; o[7] += f[u] * a1.w;
        }
        if (NS == 1) {
            attn_store_slice<HD>(o, L > 0.f ? 1.f / L : 0.f, Hq, head, t, tt, hh, lane, xhi, xlo);
        } else {
            // this range's partial: O as [(tt, hh)][register quad j][lane][4] (a wave writes 1 KB at a time), then
            // (M, L)[32 rows]
            float *pp = part + ((size_t)(t * Hq + head) * NS + split) * PF;
            store16_agent(pp + (((tt * 2 + hh) * 2 + 0) * 64 + lane) * 4, o[0], o[1], o[2], o[3]);
            store16_agent(pp + (((tt * 2 + hh) * 2 + 1) * 64 + lane) * 4, o[4], o[5], o[6], o[7]);
            if (w == 0 && half == 0) st_agent2(pp + 32 * HD + 2 * qrow, M, L);
        }
    }
    if (NS == 1) return;
    // the key range that arrives last at the head's counter merges all of them
    if (!arrive_last(counters + t * Hq + head, NS, &as.last)) { prefetch_next(nx, as.slot); return; }
    if (w < 2 * HT) attn_head_merge<HD>(part, NS, Hq, scale_log2e, xhi, xlo, head, t, w >> 1, w & 1, lane);
}

// grid: x = kv_head + Hkv * (head in group + G * split), y = pass tile; 512 threads
template <int HD>
__global__ __launch_bounds__(512) void k_attn_head(const uint4 *__restrict__ Qhi, const uint4 *__restrict__ Qlo,
                                                   const uint16_t *__restrict__ Kc, const uint16_t *__restrict__ Vt,
                                                   size_t seq_stride, size_t head_stride,
                                                   const int *__restrict__ tile_seq, const int *__restrict__ row_limit,
                                                   float *__restrict__ part, int *__restrict__ counters, int Hq, int Hkv,
                                                   int NS, float scale_log2e, uint4 *__restrict__ xhi,
                                                   uint4 *__restrict__ xlo, const NextWeights nx) {
    __shared__ __attribute__((aligned(16))) AttnHeadSmem<HD> as;
    const int t = blockIdx.y;
    const int G = Hq / Hkv, kvh = blockIdx.x % Hkv, r = blockIdx.x / Hkv;
    attn_head_item<HD>(Qhi, Qlo, Kc, Vt, seq_stride, head_stride, tile_seq[t], row_limit[t * 32 + (threadIdx.x & 31)], part,
                       counters, Hq, Hkv, NS, scale_log2e, xhi, xlo, as, kvh * G + r % G, r / G, t, nx);
}

// ------------------------------------------------------------------------------------------
// acceptance and commit, one block per sequence
// ------------------------------------------------------------------------------------------
struct AcceptOut { int *accept_len, *n_committed, *committed; };   // device [B], [B], [B][k + bonus]

// bonus = 1: the target pass had k + 1 rows and `corr` is also the extra token after k accepted drafts
__device__ __forceinline__ void commit_tokens(SeqState st, AcceptOut out, int b, int k, int a, int corr, const int *d,
                                              int eos, int bonus) {
    // thread 0 only
    const int cs = k + bonus;
    int n = (a < k) ? a + 1 : cs;
    int fin = 0;
    for (int i = 0; i < n; ++i) {
        int tok = (i < a) ? d[i] : corr;
        out.committed[b * cs + i] = tok;
        st.ing_tok[b * 32 + i] = tok;
        if (eos >= 0 && tok == eos) { n = i + 1; fin = 1; break; }
    }
    out.accept_len[b] = a;
    out.n_committed[b] = n;
    st.ing_n[b] = n;
    st.len[b] += n;
    st.pending[b] = out.committed[b * cs + n - 1];
    if (fin) st.finished[b] = 1;
}

// T = 0: accept while the draft equals the target's argmax; the first mismatch is replaced by it; with the
// bonus token on, k matches are followed by the argmax of row k
__global__ void k_accept_greedy(SeqState st, AcceptOut out, const int *__restrict__ draft,
                                const RowResult *__restrict__ tres, int k, int eos, int bonus) {
    const int b = blockIdx.x;
    if (threadIdx.x != 0) return;
    if (st.finished[b]) { out.accept_len[b] = 0; out.n_committed[b] = 0; return; }
    const int *d = draft + b * k;
    const int kt = k + bonus;
    int a = k, corr = bonus ? tres[b * kt + k].argmax : -1;
    for (int i = 0; i < k; ++i) {
        int tgt = tres[b * kt + i].argmax;
        if (d[i] != tgt) { a = i; corr = tgt; break; }
    }
    commit_tokens(st, out, b, k, a, corr, d, eos, bonus);
}

// T > 0: u_i <= min(1, p_i(y^_i) / q_i(y^_i)) in log space, stop at the first rejection and draw the
// replacement from max(0, p_i - q_i) by Gumbel-max (falls back to p_i when the residual is empty).
// With the bonus token on, k acceptances are followed by a draw from p_{k+1} (a residual without a draft:
// the same generator stream at position j + k, weights p).
// Grid (sequence, ACC_NB): every workgroup repeats the k tests (cheap), then scans its share of the vocabulary
// row; the candidates of the ACC_NB shares meet through memory and the workgroup that arrives last picks the
// winner (largest perturbed weight, lowest index on ties: the same token whatever the split) and commits.
// The kernel reads nothing that it writes before all shares have arrived: the committed length j comes from
// the verify pass's row metadata (row 0 of the sequence's tile sits at position j - 1), every share arrives
// on every path (finished sequence, all k drafts accepted, a draw), and only the last arrival touches the
// per-sequence state and resets the counter.
constexpr int ACC_NB = 32;
struct AccPart { float best; int bi; float bestp; int bpi; int any; int pad[3]; };

__global__ __launch_bounds__(1024) void k_accept_sample(SeqState st, AcceptOut out, const int *__restrict__ draft,
                                                        const RowResult *__restrict__ tres,
                                                        const RowResult *__restrict__ dres,
                                                        const float *__restrict__ tlogits,
                                                        const float *__restrict__ dlogits, int k, int V, float T,
                                                        uint64_t seed, int eos, int bonus, AccPart *parts, int *arrivals,
                                                        const int *__restrict__ verify_pos) {
    __shared__ int s_a, s_last;
    __shared__ float sv[1024]; __shared__ int sx[1024];
    __shared__ float sv2[1024]; __shared__ int sx2[1024]; __shared__ int s_any[1024];
    const int b = blockIdx.x, nb = gridDim.y, part = blockIdx.y;
    const bool finished = st.finished[b] != 0;   // written only by the last arrival, after this read
    const int *d = draft + b * k;
    const int kt = k + bonus;           // target rows per sequence
    const int j = verify_pos[b * 32] + 1;
    const float invT = 1.f / T;
    if (threadIdx.x < 64) {   // the k tests at once (each has its own uniform and rows), then the first rejection
        const int i = threadIdx.x;
        int rej = k;
        if (i < k && !finished) {
            const size_t rt = (size_t)b * kt + i, rd = (size_t)b * k + i;
            const int y = d[i];
            const float logp = tlogits[rt * V + y] * invT - tres[rt].lse;
            const float logq = dlogits[rd * V + y] * invT - dres[rd].lse;
            const float u = uniform01(row_key(seed, TAG_ACCEPT, (uint64_t)b, (uint64_t)(j + i)), 0);
            if (!(logf(u) <= fminf(0.f, logp - logq))) rej = i;
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) rej = min(rej, shx(rej, off));
        if (i == 0) s_a = rej;
    }
    __syncthreads();
    const int a = s_a;
    const bool draw = !finished && (a < k || bonus);   // a token has to be drawn (k accepted drafts without the extra token: nothing to draw)
    if (draw) {
        const bool has_q = a < k;       // a drafted token stands at this position
        const size_t rt = (size_t)b * kt + a, rd = (size_t)b * k + (has_q ? a : 0);
        const float lt = tres[rt].lse, ld = has_q ? dres[rd].lse : 0.f;
        const uint64_t key = row_key(seed, TAG_RESID, (uint64_t)b, (uint64_t)(j + a));
        float best = -INFINITY, bestp = -INFINITY; int bi = 0x7fffffff, bpi = 0x7fffffff, any = 0;
        const int share = (V + nb - 1) / nb, v0 = part * share, v1 = min(V, v0 + share);
        for (int v = v0 + threadIdx.x; v < v1; v += 1024) {
            const float logp = tlogits[rt * V + v] * invT - lt;
            const float gn = gumbel(key, (uint64_t)v);
            if (has_q) {
                const float logq = dlogits[rd * V + v] * invT - ld;
                const float diff = expf(logp) - expf(logq);
                if (diff > 0.f) { any = 1; argmax_merge(best, bi, logf(diff) + gn, v); }
            }
            argmax_merge(bestp, bpi, logp + gn, v);
        }
        s_any[threadIdx.x] = any; sv[threadIdx.x] = best; sx[threadIdx.x] = bi; sv2[threadIdx.x] = bestp; sx2[threadIdx.x] = bpi;
        __syncthreads();
        for (int off = 512; off > 0; off >>= 1) {
            if (threadIdx.x < off) {
                s_any[threadIdx.x] |= s_any[threadIdx.x + off];
                argmax_merge(sv[threadIdx.x], sx[threadIdx.x], sv[threadIdx.x + off], sx[threadIdx.x + off]);
                argmax_merge(sv2[threadIdx.x], sx2[threadIdx.x], sv2[threadIdx.x + off], sx2[threadIdx.x + off]);
            }
            __syncthreads();
        }
        if (threadIdx.x == 0) {
            AccPart *pp = parts + (size_t)b * nb + part;
            __hip_atomic_store(&pp->best, sv[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&pp->bi, sx[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&pp->bestp, sv2[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&pp->bpi, sx2[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(&pp->any, s_any[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (!arrive_last(arrivals + b, nb, &s_last)) return;
    if (threadIdx.x != 0) return;
    if (finished) { out.accept_len[b] = 0; out.n_committed[b] = 0; return; }
    int corr = -1;
    if (draw) {
        int any_all = 0;
        for (int p = 0; p < nb; ++p) any_all |= __hip_atomic_load(&parts[(size_t)b * nb + p].any, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        float wv = -INFINITY; int wi = 0x7fffffff;
        for (int p = 0; p < nb; ++p) {
            const AccPart *pp = parts + (size_t)b * nb + p;
            const float cv = __hip_atomic_load(any_all ? &pp->best : &pp->bestp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const int ci = __hip_atomic_load(any_all ? &pp->bi : &pp->bpi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            argmax_merge(wv, wi, cv, ci);
        }
        corr = (wi >= 0 && wi < V) ? wi : 0;   // all-NaN rows never update the index
    }
    commit_tokens(st, out, b, k, a, corr, d, eos, bonus);
}

// Test aid: the caller's tokens are committed in place of the acceptance rule's choice.  One thread per sequence;
// n[b] tokens tok[b * stride ..] (n[b] = 0: nothing).  Same state updates as commit_tokens.
__global__ void k_force_commit(SeqState st, const int *__restrict__ tok, const int *__restrict__ n, int stride, int eos, int B) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int nb = n[b];
    if (nb <= 0) { st.ing_n[b] = 0; return; }
    int fin = 0;
    for (int i = 0; i < nb; ++i) {
        const int t = tok[b * stride + i];
        st.ing_tok[b * 32 + i] = t;
        if (eos >= 0 && t == eos) fin = 1;
    }
    st.ing_n[b] = nb;
    st.len[b] += nb;
    st.pending[b] = tok[b * stride + nb - 1];
    if (fin) st.finished[b] = 1;
}

// Test aid: canonical K and V rows [n][kv_head][head_dim] (bf16) into cache slots first .. first + n - 1 of one
// sequence and layer.  One thread per (slot, head, channel octet).
__global__ void k_load_kv(const uint16_t *__restrict__ krows, const uint16_t *__restrict__ vrows, KvView kv, int b, int first,
                          int n, int Hkv, int hd) {
    const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int octs = hd >> 3;
    if (gid >= (size_t)n * Hkv * octs) return;
    const int oct = (int)(gid % octs), head = (int)((gid / octs) % Hkv), r = (int)(gid / ((size_t)octs * Hkv));
    const int slot = first + r;
    const size_t src = ((size_t)r * Hkv + head) * hd + oct * 8;
    const size_t base = (size_t)b * kv.seq_stride + (size_t)head * kv.head_stride;
    *(uint4 *)(kv.k + base + k_cache_off(slot, oct, hd)) = *(const uint4 *)(krows + src);
#pragma unroll
    for (int e = 0; e < 8; ++e) kv.vt[base + v_cache_off(slot, oct * 8 + e, hd)] = vrows[src + e];
}

}  // namespace deer
