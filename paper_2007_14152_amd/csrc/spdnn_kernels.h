// Device code of the spdnn library (gfx950 only, wave64).
//
// Mapping.  A workgroup of 1024 threads owns a block of 1024 consecutive output
// neurons (one per lane) for its whole life and keeps their 32 (column, weight)
// pairs in registers -- the register tiling of Section III-A-1, with the reuse
// extended from a fixed mini-batch to every feature row the workgroup walks
// over.  Feature rows stream through LDS four at a time: a tile holds, for
// every column of the block's input window, the four rows' values side by side
// (16 bytes), so one ds_read_b128 per connection feeds four FMAs -- the
// shared-memory tiling of Section III-A-2, with the preload list replaced by the
// block's contiguous column window [c_lo, c_lo + ncols).  Two tiles are kept in
// LDS (next one is loaded while the current one is used).  Windows wider than
// kCap columns are walked in kCap-column stages; a connection contributes in the
// stage its column falls in.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace spdnn {

constexpr int kNnz = 32;     // connections per output neuron
constexpr int kBlk = 1024;   // output neurons per workgroup = threads per workgroup
constexpr int kRows = 4;     // feature rows per LDS tile
constexpr int kCap = 4096;   // columns per LDS stage
constexpr int kCapLog2 = 12;
constexpr float kClip = 32.0f;

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Byte offset inside the LDS tile pair of stage-local column c, buffer 0.  The two
// buffers interleave in chunks of 8 columns (128 bytes) so that the second buffer
// is reached with a constant +128, which fits the instruction's immediate offset.
__host__ __device__ inline uint32_t tile_offset(uint32_t c) {
    return ((c >> 3) << 8) | ((c & 7u) << 4);
}

struct LayerWeights {
    const uint16_t* rel;  // [nblk][32][kBlk] column - c_lo of the block
    const float* val;     // [nblk][32][kBlk]
    const int2* win;      // [nblk] {c_lo, ncols}, both multiples of 4
};

// Eight connections of one output neuron applied to the four rows of an LDS
// tile: acc[r] = fma(tile[col_k][r], w_k, acc[r]) for k = 0..7 in that order.
// Hand-scheduled: four 16-byte LDS reads are kept in flight in v112..v127 and
// each is refilled as soon as its four FMAs have issued, so reads and FMAs of one
// wave overlap without the register blow-up the compiler's own schedule gives.
// P selects the tile buffer through the read's immediate offset.
template <int P>
__device__ __forceinline__ void fma_block8(float (&acc)[4], const uint32_t (&o)[8], const float (&w)[8]) {
#define SPDNN_FMA4(T, W)                                   \
    "v_fmac_f32 %[a0], v" #T "+0, %[" #W "]\n\t"           \
    "v_fmac_f32 %[a1], v" #T "+1, %[" #W "]\n\t"           \
    "v_fmac_f32 %[a2], v" #T "+2, %[" #W "]\n\t"           \
    "v_fmac_f32 %[a3], v" #T "+3, %[" #W "]\n\t"
    asm volatile(
        "ds_read_b128 v[112:115], %[o0] offset:%[B]\n\t"
        "ds_read_b128 v[116:119], %[o1] offset:%[B]\n\t"
        "ds_read_b128 v[120:123], %[o2] offset:%[B]\n\t"
        "ds_read_b128 v[124:127], %[o3] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], v112, %[w0]\n\t"
        "v_fmac_f32 %[a1], v113, %[w0]\n\t"
        "v_fmac_f32 %[a2], v114, %[w0]\n\t"
        "v_fmac_f32 %[a3], v115, %[w0]\n\t"
        "ds_read_b128 v[112:115], %[o4] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], v116, %[w1]\n\t"
        "v_fmac_f32 %[a1], v117, %[w1]\n\t"
        "v_fmac_f32 %[a2], v118, %[w1]\n\t"
        "v_fmac_f32 %[a3], v119, %[w1]\n\t"
        "ds_read_b128 v[116:119], %[o5] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], v120, %[w2]\n\t"
        "v_fmac_f32 %[a1], v121, %[w2]\n\t"
        "v_fmac_f32 %[a2], v122, %[w2]\n\t"
        "v_fmac_f32 %[a3], v123, %[w2]\n\t"
        "ds_read_b128 v[120:123], %[o6] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], v124, %[w3]\n\t"
        "v_fmac_f32 %[a1], v125, %[w3]\n\t"
        "v_fmac_f32 %[a2], v126, %[w3]\n\t"
        "v_fmac_f32 %[a3], v127, %[w3]\n\t"
        "ds_read_b128 v[124:127], %[o7] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], v112, %[w4]\n\t"
        "v_fmac_f32 %[a1], v113, %[w4]\n\t"
        "v_fmac_f32 %[a2], v114, %[w4]\n\t"
        "v_fmac_f32 %[a3], v115, %[w4]\n\t"
        "s_waitcnt lgkmcnt(2)\n\t"
        "v_fmac_f32 %[a0], v116, %[w5]\n\t"
        "v_fmac_f32 %[a1], v117, %[w5]\n\t"
        "v_fmac_f32 %[a2], v118, %[w5]\n\t"
        "v_fmac_f32 %[a3], v119, %[w5]\n\t"
        "s_waitcnt lgkmcnt(1)\n\t"
        "v_fmac_f32 %[a0], v120, %[w6]\n\t"
        "v_fmac_f32 %[a1], v121, %[w6]\n\t"
        "v_fmac_f32 %[a2], v122, %[w6]\n\t"
        "v_fmac_f32 %[a3], v123, %[w6]\n\t"
        "s_waitcnt lgkmcnt(0)\n\t"
        "v_fmac_f32 %[a0], v124, %[w7]\n\t"
        "v_fmac_f32 %[a1], v125, %[w7]\n\t"
        "v_fmac_f32 %[a2], v126, %[w7]\n\t"
        "v_fmac_f32 %[a3], v127, %[w7]\n\t"
        : [a0] "+v"(acc[0]), [a1] "+v"(acc[1]), [a2] "+v"(acc[2]), [a3] "+v"(acc[3])
        : [o0] "v"(o[0]), [o1] "v"(o[1]), [o2] "v"(o[2]), [o3] "v"(o[3]), [o4] "v"(o[4]), [o5] "v"(o[5]),
          [o6] "v"(o[6]), [o7] "v"(o[7]), [w0] "v"(w[0]), [w1] "v"(w[1]), [w2] "v"(w[2]), [w3] "v"(w[3]),
          [w4] "v"(w[4]), [w5] "v"(w[5]), [w6] "v"(w[6]), [w7] "v"(w[7]), [B] "n"(P * 128)
        : "v112", "v113", "v114", "v115", "v116", "v117", "v118", "v119", "v120", "v121", "v122", "v123",
          "v124", "v125", "v126", "v127", "memory");
#undef SPDNN_FMA4
}

// ---------------------------------------------------------------------------
// a1: fused SpMM + bias + clipped ReLU for one layer (Eq. 1), plus the per-row
// "has a positive output" flag that Listings 1 and 2 keep in active[].
//
// Yin is read through cat[] (slot of every active row in the buffer written by
// the previous layer); row i of the active list is written to slot i of Yout.
// *count_ptr = number of active rows A.  The grid is nblk * G-aligned units
// (see unit mapping below); a workgroup handles row groups
// [q*per, (q+1)*per) of ceil(A/4).
// ---------------------------------------------------------------------------
template <bool MULTI>
__global__ __launch_bounds__(kBlk) void fused_layer_kernel(
    const float* __restrict__ Yin, const int* __restrict__ cat, float* __restrict__ Yout,
    int* __restrict__ flags, const int* __restrict__ count_ptr, LayerWeights w,
    const float* __restrict__ bias, int N, int nblk, int G, int Q) {
    extern __shared__ float4 lds4[];
    const int tid = threadIdx.x;

    // Workgroup -> (output block b, row chunk q).  Consecutive workgroup ids go to
    // consecutive XCDs (8 of them, each with its own L2).  The G output blocks that
    // read the same rows through overlapping windows form a unit; a unit's
    // workgroups are given ids that are equal modulo 8, so they share one L2.
    const int xcd = blockIdx.x & 7;
    const int slot = blockIdx.x >> 3;
    const int unit = (slot / G) * 8 + xcd;
    const int sub = slot - (slot / G) * G;
    const int ngrp = nblk / G;
    if (unit >= ngrp * Q) return;
    const int q = unit / ngrp;
    const int b = (unit - q * ngrp) * G + sub;

    const int A = *count_ptr;
    const int ngroups = (A + kRows - 1) / kRows;
    const int per = (ngroups + Q - 1) / Q;
    const int g0 = q * per;
    const int g1 = min(ngroups, g0 + per);
    if (g0 >= g1) return;

    const int j = b * kBlk + tid;
    const bool jok = j < N;
    const int2 win = w.win[b];
    const int c_lo = win.x;
    const int ncols = win.y;
    const int nstage = MULTI ? (ncols + kCap - 1) / kCap : 1;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds4;  // LDS byte address of the tile pair

    // Connections of my output neuron, in registers for the whole kernel.
    // off = LDS byte address (buffer 0) of the column inside its stage; MULTI also
    // keeps the stage number in bits 20 and up.
    uint32_t off[kNnz];
    float wv[kNnz];
    {
        const uint16_t* prel = w.rel + (size_t)b * kNnz * kBlk + tid;
        const float* pval = w.val + (size_t)b * kNnz * kBlk + tid;
#pragma unroll
        for (int k = 0; k < kNnz; ++k) {
            const uint32_t rel = prel[k * kBlk];
            wv[k] = pval[k * kBlk];
            if (MULTI)
                off[k] = (lds_base + tile_offset(rel & (kCap - 1))) | ((rel >> kCapLog2) << 20);
            else
                off[k] = lds_base + tile_offset(rel);
        }
    }
    const float bj = jok ? bias[j] : 0.0f;

    const int T = (g1 - g0) * nstage;  // pipeline steps: (row group, stage) pairs
    // Staging: lane owns columns tid, tid+1024, tid+2048, tid+3072 of the stage; for
    // each it fetches the 4 rows (4 coalesced dword loads per row across the wave)
    // and writes them to LDS as one 16-byte entry.
    float4 st[4];
    const uint32_t st_addr = lds_base + tile_offset(tid);  // + i*32768 for column tid + 1024 i

    auto load_tile = [&](int t) {
        const int gi = MULTI ? t / nstage : t;
        const int s = MULTI ? t - gi * nstage : 0;
        const float* rowp[kRows];
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const int row = min((g0 + gi) * kRows + r, A - 1);
            rowp[r] = Yin + (size_t)cat[row] * N + c_lo + s * kCap;
        }
        const int left = ncols - s * kCap;  // columns in this stage (may exceed kCap)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = tid + i * kBlk;
            if (c < left) {
                st[i].x = rowp[0][c];
                st[i].y = rowp[1][c];
                st[i].z = rowp[2][c];
                st[i].w = rowp[3][c];
            }
        }
    };
    auto store_tile = [&](int P, int t) {
        const int gi = MULTI ? t / nstage : t;
        const int s = MULTI ? t - gi * nstage : 0;
        const int left = ncols - s * kCap;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c = tid + i * kBlk;
            if (c < left)
                *reinterpret_cast<__attribute__((address_space(3))) f32x4*>(st_addr + i * 32768 + P * 128) =
                    f32x4{st[i].x, st[i].y, st[i].z, st[i].w};
        }
    };

    float acc[kRows] = {0.f, 0.f, 0.f, 0.f};

    auto compute = [&](auto Ptag, int s) {
        constexpr int P = decltype(Ptag)::value;
#pragma unroll
        for (int k0 = 0; k0 < kNnz; k0 += 8) {
            uint32_t o[8];
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                o[i] = off[k0 + i];
                v[i] = wv[k0 + i];
                if (MULTI) {
                    // a connection outside this stage reads column 0 of the stage (always
                    // loaded) with weight 0: adds exactly 0 for finite features
                    const bool mine = (int)(o[i] >> 20) == s;
                    o[i] = mine ? (o[i] & 0xFFFFFu) : lds_base;
                    v[i] = mine ? v[i] : 0.0f;
                }
            }
            fma_block8<P>(acc, o, v);
        }
    };

    auto epilogue = [&](int g) {
#pragma unroll
        for (int r = 0; r < kRows; ++r) {
            const int row = g * kRows + r;
            const float z = acc[r] + bj;
            const float y = fminf(fmaxf(z, 0.0f), kClip);
            const bool live = jok && row < A;
            if (live) Yout[(size_t)row * N + j] = y;
            const unsigned long long m = __ballot(live && y > 0.0f);
            if (m != 0ull && (tid & 63) == 0) flags[row] = 1;
            acc[r] = 0.0f;
        }
    };

    // One pipeline step with compile-time buffer index P.
    auto step = [&](int t, auto Ptag) {
        constexpr int P = decltype(Ptag)::value;
        const bool more = t + 1 < T;
        if (more) load_tile(t + 1);
        const int gi = MULTI ? t / nstage : t;
        const int s = MULTI ? t - gi * nstage : 0;
        compute(Ptag, s);
        if (s == nstage - 1) epilogue(g0 + gi);
        if (more) store_tile(P ^ 1, t + 1);
        __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;

    load_tile(0);
    store_tile(0, 0);
    __syncthreads();
    int t = 0;
    for (; t + 1 < T; t += 2) {
        step(t, P0{});
        step(t + 1, P1{});
    }
    if (t < T) step(t, P0{});
}

// ---------------------------------------------------------------------------
// a2: active-row compaction (the host loop of Listing 1 between two layers,
// moved onto the GPU).  Stable filter of the A rows whose flag is set:
// cat_out[p] = slot in the buffer just written, gid_out[p] = original row id,
// *count = new A; flags are cleared for the next layer.  One workgroup; per
// 1024-row chunk a wave64 ballot + popcount gives the rank inside the wave and
// the 16 wave totals are combined through LDS.  The new count is also stored to
// pinned host memory so the host can size later launches without a stream sync.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void compact_kernel(int* __restrict__ flags, int* __restrict__ count,
                                                       const int* __restrict__ gid_in,
                                                       int* __restrict__ gid_out, int* __restrict__ cat_out,
                                                       int* host_count) {
    __shared__ int wsum[16];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int A = *count;
    int base = 0;
    for (int start = 0; start < A; start += 1024) {
        const int i = start + tid;
        int f = 0, g = 0;
        if (i < A) {
            f = flags[i];
            g = gid_in[i];
            flags[i] = 0;
        }
        const unsigned long long m = __ballot(f != 0);
        const int prefix = __popcll(m & ((1ull << lane) - 1ull));
        if (lane == 0) wsum[wave] = __popcll(m);
        __syncthreads();
        int woff = 0, total = 0;
#pragma unroll
        for (int wv = 0; wv < 16; ++wv) {
            const int c = wsum[wv];
            woff += (wv < wave) ? c : 0;
            total += c;
        }
        if (f != 0) {
            const int p = base + woff + prefix;
            cat_out[p] = i;
            gid_out[p] = g;
        }
        base += total;
        __syncthreads();
    }
    if (tid == 0) {
        *count = base;
        __hip_atomic_store(host_count, base, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

// Start of an inference: identity lists, cleared flags, A = batch.
__global__ void init_lists_kernel(int* __restrict__ cat, int* __restrict__ gid, int* __restrict__ flags,
                                  int* __restrict__ count, int batch) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < batch) {
        cat[i] = i;
        gid[i] = i;
        flags[i] = 0;
    }
    if (i == 0) *count = batch;
}

// a4: surviving rows of Y_L, gathered into a dense [n][N] array (16-byte pieces).
__global__ void gather_rows_kernel(const float4* __restrict__ src, const int* __restrict__ cat, int n,
                                   int n4, float4* __restrict__ dst) {
    const size_t total = (size_t)n * n4;
    for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total;
         e += (size_t)gridDim.x * blockDim.x) {
        const size_t row = e / n4;
        const size_t c = e - row * n4;
        dst[e] = src[(size_t)cat[row] * n4 + c];
    }
}

// ---------------------------------------------------------------------------
// a0 (set-up): per output block, the column window its connections span, then the
// lane-major copy of the connections (consecutive lanes read consecutive
// addresses, as the transposed sliced-ELL of Section III-A-3 is meant to give).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlk) void block_window_kernel(const int32_t* __restrict__ idx, int N,
                                                            int2* __restrict__ win, int* __restrict__ err) {
    __shared__ int s_lo, s_hi;
    const int tid = threadIdx.x;
    const int j = blockIdx.x * kBlk + tid;
    if (tid == 0) {
        s_lo = N;
        s_hi = -1;
    }
    __syncthreads();
    int lo = N, hi = -1;
    if (j < N) {
        for (int k = 0; k < kNnz; ++k) {
            const int c = idx[(size_t)j * kNnz + k];
            if (c < 0 || c >= N) {
                *err = 1;
            } else {
                lo = min(lo, c);
                hi = max(hi, c);
            }
        }
    }
    atomicMin(&s_lo, lo);
    atomicMax(&s_hi, hi);
    __syncthreads();
    if (tid == 0) {
        int c_lo = 0, ncols = 4;
        if (s_hi >= s_lo) {
            c_lo = s_lo & ~3;
            ncols = ((s_hi + 1 - c_lo) + 3) & ~3;
        }
        win[blockIdx.x] = make_int2(c_lo, ncols);
    }
}

__global__ __launch_bounds__(kBlk) void pack_weights_kernel(const int32_t* __restrict__ idx,
                                                            const float* __restrict__ val, int N,
                                                            const int2* __restrict__ win,
                                                            uint16_t* __restrict__ rel,
                                                            float* __restrict__ wval) {
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    const int j = b * kBlk + tid;
    const int c_lo = win[b].x;
    for (int k = 0; k < kNnz; ++k) {
        const size_t e = ((size_t)b * kNnz + k) * kBlk + tid;
        int c = c_lo;
        float v = 0.0f;
        if (j < N) {
            c = idx[(size_t)j * kNnz + k];
            v = val[(size_t)j * kNnz + k];
            if (c < 0 || c >= N) {  // reported by block_window_kernel; keep the copy in range
                c = c_lo;
                v = 0.0f;
            }
        }
        rel[e] = (uint16_t)(c - c_lo);
        wval[e] = v;
    }
}

}  // namespace spdnn
