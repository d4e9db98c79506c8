// Device-side building blocks shared by the gfx950 kernels: MFMA fragment helpers, coalesced
// global->LDS tile loaders, and the per-sequence draft-tree metadata (Section 2.1, Section 4.1).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ssv {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;   // 4 wavefronts of 64 lanes
constexpr int kTile = 64;       // KV rows per streamed tile (= one selection block)
constexpr int kMaxT = 128;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// One "fragment" is 16 bytes of a row: 8 bf16 or 4 fp32 values of the contraction dimension.
// A 64-byte chunk of every row is spread over the four 16-lane groups of a wavefront
// (group G = lane / 16 holds bytes [16 G, 16 G + 16)), and both MFMA operands use the same
// assignment, so the contraction runs over the whole chunk whatever order the hardware
// enumerates it in.  Result layout of every 16x16 MFMA: lane (n = lane % 16, G) holds
// D[4 G + r][n], r = 0..3.
template <bool BF16>
__device__ __forceinline__ f32x4 mma_frag(u32x4 a, u32x4 b, f32x4 c) {
    if constexpr (BF16) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c,
                                                       0, 0, 0);
    } else {
        f32x4 af = __builtin_bit_cast(f32x4, a), bf = __builtin_bit_cast(f32x4, b);
#pragma unroll
        for (int j = 0; j < 4; ++j) c = __builtin_amdgcn_mfma_f32_16x16x4f32(af[j], bf[j], c, 0, 0, 0);
        return c;
    }
}

// Wait until at most N of this wavefront's vector memory loads are outstanding (they return in order).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | 0x0F70 | ((N >> 4) << 14));   // expcnt and lgkmcnt fields left at "no wait"
}

// The same for a wave-uniform run-time count (a branch tree over the immediates); counts of 32 and more wait for 31.
__device__ __forceinline__ void wait_vmcnt_upto(int n) {
    n = __builtin_amdgcn_readfirstlane(n);
#define SSV_W4(b) \
    switch (n & 3) { case 0: wait_vmcnt<(b)>(); break; case 1: wait_vmcnt<(b) + 1>(); break; \
                     case 2: wait_vmcnt<(b) + 2>(); break; default: wait_vmcnt<(b) + 3>(); break; }
    if (n >= 32) { wait_vmcnt<31>(); return; }
    switch (n >> 2) {
        case 0: SSV_W4(0) break;
        case 1: SSV_W4(4) break;
        case 2: SSV_W4(8) break;
        case 3: SSV_W4(12) break;
        case 4: SSV_W4(16) break;
        case 5: SSV_W4(20) break;
        case 6: SSV_W4(24) break;
        default: SSV_W4(28) break;
    }
#undef SSV_W4
}

// Exchange with the lane 16 (32) positions away, without going through LDS: the gfx950 swap instructions return
// the operand with its odd 16-lane (upper 32-lane) rows replaced by the even (lower) ones, and the reverse, so
// combining the two results leaves op(x[l], x[l ^ 16]) (op(x[l], x[l ^ 32])) in every lane.
// Maximum of two floats with the NaN-propagating instruction (v_maximum3_f32 on gfx950): unlike the IEEE maximum it
// needs no canonicalisation of its inputs (one extra instruction per matrix-instruction result under the default
// floating-point mode), and two nested calls fuse into one three-operand instruction.  Equal to fmaxf for non-NaN inputs.
__device__ __forceinline__ float max_nan(float a, float b) { return __builtin_elementwise_maximum(a, b); }

__device__ __forceinline__ float xor16_max(float x) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return max_nan(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xor32_max(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return max_nan(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xor16_add(float x) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float xor32_add(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ u32x4 lds_read16(const char* p) { return *reinterpret_cast<const u32x4*>(p); }
__device__ __forceinline__ u32x2 lds_read8(const char* p) { return *reinterpret_cast<const u32x2*>(p); }
// LDS addresses as 32-bit integers (for address arithmetic that pointers do not allow, such as XOR)
__device__ __forceinline__ uint32_t lds_addr(const char* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}
__device__ __forceinline__ u32x4 lds_read16_at(uint32_t addr) {
    return *reinterpret_cast<__attribute__((address_space(3))) const u32x4*>((uintptr_t)addr);
}

// Tile loaders come in two halves so that the global loads of the next tile can be in flight while the
// current tile is being computed: *_issue reads into registers, *_commit writes the registers to LDS.
// All global loads are unconditional (the row index is clamped, the value is zeroed at commit), so they
// are issued back to back and wait once; a predicated load would serialise on its branch.
// Rows >= valid_rows (>= 1) are zero-filled: their memory may not exist or may hold non-finite values.

// Row-major copy of up to 64 rows of ROW_BYTES bytes into LDS with row pitch PITCH.
template <int ROW_BYTES>
struct RowTileRegs {
    static constexpr int CPR = ROW_BYTES / 16;
    static constexpr int TOTAL = kTile * CPR;
    static_assert(TOTAL % kThreads == 0, "tile must divide evenly over the workgroup");
    static constexpr int ITERS = TOTAL / kThreads;
    u32x4 val[ITERS];
    uint32_t off[ITERS];     // byte offsets of this thread's chunks inside a full tile (tile-invariant)

    __device__ __forceinline__ void init(uint32_t g_row_bytes, int tid) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int f = it * kThreads + tid;
            off[it] = (uint32_t)(f / CPR) * g_row_bytes + (uint32_t)(f % CPR) * 16u;
        }
    }
    __device__ __forceinline__ void issue(const char* g, uint32_t g_row_bytes, int valid_rows, int tid) {
        if (valid_rows == kTile) {           // uniform; every tile but the last one of a sequence
#pragma unroll
            for (int it = 0; it < ITERS; ++it) val[it] = *reinterpret_cast<const u32x4*>(g + off[it]);
        } else {
            const int last = valid_rows - 1;
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                const int f = it * kThreads + tid;
                const int row = f / CPR, col = f % CPR;
                val[it] = *reinterpret_cast<const u32x4*>(g + (uint32_t)min(row, last) * g_row_bytes + (uint32_t)col * 16u);
            }
        }
    }
    template <int PITCH>
    __device__ __forceinline__ void commit(char* lds, int valid_rows, int tid) {
        if (valid_rows < kTile) {            // uniform; rare
#pragma unroll
            for (int it = 0; it < ITERS; ++it)
                if ((it * kThreads + tid) / CPR >= valid_rows) val[it] = u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int f = it * kThreads + tid;
            const int row = f / CPR, col = f % CPR;
            *reinterpret_cast<u32x4*>(lds + row * PITCH + col * 16) = val[it];
        }
    }
};

// Row-major tile of 64 rows x ROW_BYTES brought from global memory straight into LDS (gfx950 16-byte
// buffer->LDS loads: the 64 lanes of one instruction fill 1 KB of LDS linearly from a wave-uniform base, each lane
// from its own offset into the buffer), no registers and no LDS store instructions in between.  Buffer loads
// rather than global ones: a global (flat-encoded) LDS load also counts as a possible LDS access of the flat
// kind, which makes the compiler wait for ALL outstanding LDS reads before every use while one is in flight.  The LDS image has no row
// padding; instead the 16-byte granule index inside every group of eight granules is XORed with the low three bits
// of the row, which spreads the sixteen rows an MFMA operand read touches over the banks as padding would.
//   granule (row r, column c)  ->  LDS granule r * CPR + swizzled(r, c), by policy SWZ:
//   0: (c & ~7) | ((c & 7) ^ (r & 7)): for operand reads in which 16 lanes take the same granule of 16 consecutive rows
//      while the other lane groups take the neighbouring granules (the 16x16x32 fragments);
//   1: (c & ~7) | ((c & 7) ^ ((r >> 1) & 7)): for reads in which 32 lanes take the same granule of 32 consecutive rows
//      (the 32x32x16 fragments: with policy 0 rows r and r + 8 of a 384- or 128-byte row pitch fall on the same banks
//      and every read is served in two passes; measured on the device);
//   2: the 64-byte chunk index c / 4 XORed with r & 3 (rows of four chunks) or (r >> 1) & 1 (rows of two): for the
//      transposing 8-byte reads of a 32x32x16 A operand, in which each half of the wavefront takes 64 bytes of four
//      consecutive rows (measured: as fast as a linear read; with an unswizzled 256-byte pitch three times slower).
// Rows beyond valid_rows repeat the last valid row (the caller masks their scores; nothing is zero-filled).
// NT: threads of the workgroup that share the tile's loads.
template <int ROW_BYTES, int SWZ = 0, int NT = kThreads>
struct DirectRowTile {
    static constexpr int CPR = ROW_BYTES / 16;            // granules per row
    static_assert(SWZ == 2 ? (CPR == 8 || CPR == 16) : CPR % 8 == 0, "row length not covered by the swizzle");
    __host__ __device__ __forceinline__ static constexpr int swizzled(int r, int c) {
        if constexpr (SWZ == 0) return (c & ~7) | ((c & 7) ^ (r & 7));
        else if constexpr (SWZ == 1) return (c & ~7) | ((c & 7) ^ ((r >> 1) & 7));
        else return (((c >> 2) ^ (CPR == 16 ? (r & 3) : ((r >> 1) & 1))) << 2) | (c & 3);
    }
    static constexpr int TOTAL = kTile * CPR;
    static_assert(TOTAL % NT == 0, "tile must divide evenly over the workgroup");
    static constexpr int ITERS = TOTAL / NT;        // load instructions per wavefront
    static constexpr int BYTES = kTile * ROW_BYTES;
    uint32_t off[ITERS];     // global byte offset, inside a full tile, of the granule this lane fetches in instruction it

    // LDS granule handled by (wave, it, lane): instruction `it` of wavefront `wave` fills granules [(wave*ITERS+it)*64, +64)
    __device__ __forceinline__ static void where(int tid, int it, int& r, int& c) {
        const int p = ((tid >> 6) * ITERS + it) * 64 + (tid & 63);
        r = p / CPR;
        const int csw = p % CPR;
        c = swizzled(r, csw);     // (the swizzle is its own inverse)
    }
    __device__ __forceinline__ void init(uint32_t g_row_bytes, int tid) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            int r, c;
            where(tid, it, r, c);
            off[it] = (uint32_t)r * g_row_bytes + (uint32_t)c * 16u;
        }
    }
    // rsrc: buffer resource over the rows of one (sequence, KV head); tile_off: byte offset of the tile's first row
    // RECOMPUTE: the (row, column) pairs behind the clamped offsets of a partial tile are derived again at every
    // partial tile instead of being kept in registers across the caller's loops (for kernels short of registers).
    template <bool RECOMPUTE = false>
    __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rsrc, uint32_t tile_off, char* lds_tile, uint32_t g_row_bytes,
                                          int valid_rows, int tid) {
        char* dst = lds_tile + (tid >> 6) * ITERS * 1024;     // wave-uniform
        if constexpr (RECOMPUTE) {
            if (valid_rows < kTile) asm volatile("" : "+v"(tid));    // opaque from here on: nothing below can be hoisted
        }
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            uint32_t o = off[it];
            if (valid_rows < kTile) {        // uniform; only the last tile of a sequence
                int r, c;
                where(tid, it, r, c);
                o = (uint32_t)min(r, valid_rows - 1) * g_row_bytes + (uint32_t)c * 16u;
            }
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void*)(dst + it * 1024), 16,
                                                     (int)o, (int)tile_off, 0, 0);
        }
    }
    // Raw buffer resource (stride 0, bounds in bytes) over `bytes` bytes at `base`: loads past the end return zero
    // instead of faulting.
    __device__ __forceinline__ static __amdgpu_buffer_rsrc_t make_rsrc(const char* base, int64_t bytes) {
        return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base), 0, (int)min(bytes, (int64_t)0x7fffffff), 0x00020000);
    }
    // byte offset, inside the tile, of granule column c0 + (kc ^ ...) handled through two per-lane bases: a lane that
    // reads row `row` and granule G of 64-byte chunk kc finds it at base(kc & 1) + kc * 64, with
    //   base(0) = row * ROW_BYTES + ((G ^ (row & 3)) * 16) + ((row >> 2) & 1) * 64,   base(1) = base(0) - 2 * ((row >> 2) & 1) * 64
    __device__ __forceinline__ static int read_base(int row, int G, int odd) {
        static_assert(SWZ == 0, "written for the row & 7 swizzle");
        const int hb = (row >> 2) & 1;
        return row * ROW_BYTES + ((G ^ (row & 3)) * 16) + (odd ? -hb * 64 : hb * 64);
    }
};

// Transposing LDS read of gfx950 (ds_read_b64_tr_b16), per group of 16 lanes: the 16 lanes supply the addresses of
// sixteen 8-byte chunks (4 bf16 each); lane i of the group receives element (i & 3) of the chunks supplied by lanes
// (i >> 2), (i >> 2) + 4, + 8, + 12 (measured on the device).  With lane i pointing at key row (i >> 2) of four
// consecutive keys, 8-byte column chunk (i & 3) of a 16-column tile, lane n receives column n of the four keys: the
// A operand of O^T = V^T P^T straight from a row-major V tile.
__device__ __forceinline__ u32x2 lds_read_tr16(const char* p) {
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
    return __builtin_bit_cast(u32x2, v);
}

__device__ __forceinline__ u32x2 lds_read_tr16_at(uint32_t addr) {
    typedef short s16x4 __attribute__((ext_vector_type(4)));
    const s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)addr);
    return __builtin_bit_cast(u32x2, v);
}

// A V tile on its way from global memory to LDS: 64 rows x DV values, staged in registers for one tile step.  Each
// work item reads four consecutive key rows of one 16-byte column chunk.  bf16 tiles are stored as they are
// (commit_rows) and transposed by the LDS reads; fp32 tiles are transposed here (commit): LDS rows indexed by the
// value column, each holding the 64 keys contiguously (pitch PITCH), one 16-byte store per column and key quad.
template <bool BF16, int DV>
struct TransposedTileRegs {
    static constexpr int ES = BF16 ? 2 : 4;
    static constexpr int CPR = DV * ES / 16;           // 16-byte chunks per row
    static constexpr int ITEMS = (kTile / 4) * CPR;    // (key quad, chunk) pairs
    static_assert(ITEMS % kThreads == 0 || kThreads % ITEMS == 0, "unsupported value width");
    static constexpr int ITERS = (ITEMS + kThreads - 1) / kThreads;
    u32x4 r[ITERS][4];
    uint32_t off[ITERS];     // byte offset of the first of this thread's four rows inside a full tile

    __device__ __forceinline__ void init(uint32_t g_row_bytes, int tid) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int item = it * kThreads + tid;
            off[it] = (uint32_t)(4 * (item / CPR)) * g_row_bytes + (uint32_t)(item % CPR) * 16u;
        }
    }
    __device__ __forceinline__ void issue(const char* g, uint32_t g_row_bytes, int valid_rows, int tid) {
        if (ITEMS < kThreads && tid >= ITEMS) return;   // whole wavefronts drop out (ITEMS is a multiple of 64)
        if (valid_rows == kTile) {           // uniform; every tile but the last one of a sequence
#pragma unroll
            for (int it = 0; it < ITERS; ++it)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    r[it][j] = *reinterpret_cast<const u32x4*>(g + off[it] + (uint32_t)j * g_row_bytes);
        } else {
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                const int item = it * kThreads + tid;
                const int kq = item / CPR, ch = item % CPR;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t o = (uint32_t)min(4 * kq + j, valid_rows - 1) * g_row_bytes + (uint32_t)ch * 16u;
                    r[it][j] = *reinterpret_cast<const u32x4*>(g + o);
                }
            }
        }
    }
    // The rows as they are (bf16): row r at r * PITCH, for the transposing LDS reads of gfx950 (vt_read_tr below).
    // PITCH is the row plus 32 bytes, which spreads the eight rows one read pass touches over all banks.
    template <int PITCH>
    __device__ __forceinline__ void commit_rows(char* lds, int valid_rows, int tid) {
        static_assert(BF16 && PITCH == DV * 2 + 32, "row-major V tile: bf16 only, padded pitch");
        if (ITEMS < kThreads && tid >= ITEMS) return;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int item = it * kThreads + tid;
            const int kq = item / CPR, ch = item % CPR;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                u32x4 v = r[it][j];
                if (valid_rows < kTile && 4 * kq + j >= valid_rows) v = u32x4{0, 0, 0, 0};   // uniform test first; rare
                *reinterpret_cast<u32x4*>(lds + (4 * kq + j) * PITCH + ch * 16) = v;
            }
        }
    }
    template <int PITCH>
    __device__ __forceinline__ void commit(char* lds, int valid_rows, int tid) {
        if (ITEMS < kThreads && tid >= ITEMS) return;
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const int item = it * kThreads + tid;
            const int kq = item / CPR, ch = item % CPR;
            if (valid_rows < kTile) {        // uniform; rare
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (4 * kq + j >= valid_rows) r[it][j] = u32x4{0, 0, 0, 0};
            }
            static_assert(!BF16, "bf16 tiles stay row-major (commit_rows)");
            {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const u32x4 o = {r[it][0][e], r[it][1][e], r[it][2][e], r[it][3][e]};
                    *reinterpret_cast<u32x4*>(lds + (ch * 4 + e) * PITCH + kq * 16) = o;
                }
            }
        }
    }
};

// Number of compressed rows a query may use: complete windows inside the contiguous visible
// extent E = L + (leading run of visible draft slots), capped by the rows that exist.
// Set of draft tokens (flattened indices 0..127): a query's ancestors and itself.
struct AncSet {
    uint64_t lo, hi;     // tokens 0..63, 64..127
};

__device__ __forceinline__ int visible_cmp_rows(AncSet anc, int L, int n_cmp, int l, int d) {
    const int lead = (~anc.lo != 0ull) ? __builtin_ctzll(~anc.lo) : 64 + ((~anc.hi != 0ull) ? __builtin_ctzll(~anc.hi) : 64);
    const int E = L + lead;
    const int full = E >= l ? (E - l) / d + 1 : 0;
    return min(full, n_cmp);
}

// Draft-tree metadata of one sequence, rebuilt by every workgroup from the parent indices:
// ancestor bitmask (bit t set iff draft token t is the query itself or one of its ancestors),
// depth (position = L + depth) and the number of compressed rows the query may use.
// parents == nullptr means a linear chain.
struct SeqMeta {
    int L, Tq, n_cmp;
};

// Lengths read from device memory are clamped to the host-side bounds every buffer and grid was sized with, so that
// an inconsistent length array cannot take a load past the end of a cache.
__device__ __forceinline__ SeqMeta build_tree_meta(int tid, int b, int T, const int32_t* seq_lens, const int32_t* n_query,
                                                   const int32_t* n_cmp, const int32_t* parents, int l, int d, int max_seq_len,
                                                   int max_n_cmp, int* s_par, int* s_depth, int* s_cmax, AncSet* s_anc) {
    SeqMeta sm;
    sm.L = min(max(seq_lens[b], 0), max_seq_len);
    sm.Tq = n_query ? min(max(n_query[b], 0), T) : T;
    sm.n_cmp = min(max(n_cmp[b], 0), max_n_cmp);
    if (parents) {
        if (tid < kMaxT) {
            int par = -1;
            if (tid < sm.Tq) {
                par = parents[(int64_t)b * T + tid];
                if (par >= tid || par < -1) par = -1;   // malformed entry: treat as a child of the prefix
            }
            s_par[tid] = par;
        }
        __syncthreads();
    }
    if (tid < kMaxT) {
        AncSet anc = {0ull, 0ull};
        int dep = 0;
        if (tid < sm.Tq) {
            if (!parents) {
                anc.lo = (tid >= 63) ? ~0ull : ((2ull << tid) - 1ull);
                anc.hi = (tid < 64) ? 0ull : ((tid == 127) ? ~0ull : ((2ull << (tid - 64)) - 1ull));
                dep = tid;
            } else {
                int t = tid;
                while (t >= 0) {        // strictly decreasing: at most tid + 1 steps
                    if (t < 64) anc.lo |= 1ull << t; else anc.hi |= 1ull << (t - 64);
                    const int pn = s_par[t];
                    if (pn >= 0) ++dep;
                    t = pn;
                }
            }
        }
        s_anc[tid] = anc;
        s_depth[tid] = dep;
        s_cmax[tid] = tid < sm.Tq ? visible_cmp_rows(anc, sm.L, sm.n_cmp, l, d) : 0;
    }
    __syncthreads();
    return sm;
}

// Representative of the verifier queries [m0, m1) of one sequence for the approximate shared-index variant
// (Section 4.3): the member with the longest prefix, i.e. the deepest one, the last of equally deep members.
__device__ __forceinline__ int group_representative(const int* s_depth, int m0, int m1) {
    int best = m0;
    for (int m = m0 + 1; m < m1; ++m)
        if (s_depth[m] >= s_depth[best]) best = m;
    return best;
}

}  // namespace ssv
