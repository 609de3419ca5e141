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

#include "spdnn_order.h"
#include "spdnn_layout.h"

namespace spdnn {

constexpr int kNnz = 32;     // connections per output neuron
constexpr int kBlk = 1024;   // output neurons per workgroup = threads per workgroup
constexpr int kRows = 4;     // feature rows per LDS tile
constexpr int kCap = 4096;   // columns per LDS stage
constexpr int kCapLog2 = 12;
constexpr float kClip = 32.0f;

typedef float f32x4 __attribute__((ext_vector_type(4)));

struct LayerWeights {
    const uint16_t* rel;  // [nblk][32][kBlk] stage << 12 | LDS slot of (column - c_lo) within the stage
    const float* val;     // [nblk][32][kBlk]
    const int2* win;      // [nblk] {c_lo, ncols}, both multiples of 4
    const uint32_t* qsel;  // [nblk][kBlk] balanced single-stage layers: see balance_kernel
};

// Layout for layers whose column windows need 3 or more LDS stages ("wide" layers).
// Connections are grouped by stage; stage s of a block offers S steps (16, or 8 when
// there are more than 8 stages); a neuron's connections of that stage fill some of
// them, the rest carry weight 0.  The few connections that do not fit (more than S
// in one stage) are kept in a spill list and gathered straight from global memory.
constexpr int kChunk = 8;  // row groups whose accumulators a workgroup keeps while it walks the stages
constexpr int kSpill = 4;  // spilled connections a neuron may have
struct WideWeights {
    const uint2* pk;            // [nblk][nstage][S/2][kBlk][2] {LDS slot of the column inside its stage, weight bits}:
                                // a lane's two consecutive steps are one 16-byte load
    const uint8_t* nb8;         // [nblk][nstage][16] blocks of 8 steps wave w needs in stage s
    const uint16_t* spill_col;  // [nblk][kSpill][kBlk] column - c_lo of a spilled connection
    const float* spill_val;     // [nblk][kSpill][kBlk] its weight (0 = none)
    const uint8_t* spill_n;     // [nblk][16] most spilled connections of any lane of wave w
    const int2* win;            // [nblk] {c_lo, ncols}
    int nstage;
    const uint4* ps;            // [nblk][nstage][S/8][kBlk] eight 16-bit LDS slots (0xFFFF = none) per 16-byte load:
                                // the compact form fused_wide_pair_kernel reads (layers with a single weight value)
    const uint16_t* sp16;       // [nblk][kSpill][kBlk] spilled connections as stage << 14 | (LDS tile byte offset >> 4)
                                // (0xFFFF = none), for fused_wide_pair4_kernel
};
constexpr int kChunkPair = 4;        // row groups per chunk when a lane holds two neurons
// Compact step lists (layers with one weight value): a 16-bit code is the LDS slot of the step's
// column, or -- for a step that pads a short list -- kPadSlot | q: "read zeros from bank quad q".
// The set-up (wide_pack_kernel) gives every padded step a quad that the other lanes served in the
// same clock do not read, so padding never collides with a real read.  The kernels keep 16 all-zero
// entries, one per quad, right behind the tile pair, where slots kCap .. kCap+15 fall (512 bytes,
// so that the second buffer's +256 lands on zeros too): padding needs no special case in them.
constexpr uint32_t kPadSlot = kCap;
// Steps per stage of the wide format: 2 stages exist only for layers that run two neurons per
// lane with all their steps in registers (2 x 32 = 4 x 16 = 64 steps per neuron).
__host__ __device__ inline int wide_steps(int nstage) { return nstage > 8 ? 8 : nstage <= 2 ? 32 : 16; }

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
          [w4] "v"(w[4]), [w5] "v"(w[5]), [w6] "v"(w[6]), [w7] "v"(w[7]), [B] "n"(P * kBufSkew)
        : "v112", "v113", "v114", "v115", "v116", "v117", "v118", "v119", "v120", "v121", "v122", "v123",
          "v124", "v125", "v126", "v127", "memory");
#undef SPDNN_FMA4
}

// Sixteen connections of one output neuron whose layer has one weight for all its
// connections (held in a scalar register): acc[r] = fma(tile[col_k][r], w, acc[r]),
// k = 0..15 in that order, four 16-byte LDS reads in flight throughout.
template <int P>
__device__ __forceinline__ void fma_block16s(float (&acc)[4], const uint32_t (&o)[16], float w) {
    asm volatile(
        "ds_read_b128 v[112:115], %[o0] offset:%[B]\n\t"
        "ds_read_b128 v[116:119], %[o1] offset:%[B]\n\t"
        "ds_read_b128 v[120:123], %[o2] offset:%[B]\n\t"
        "ds_read_b128 v[124:127], %[o3] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v112\n\t"
        "v_fmac_f32 %[a1], %[w], v113\n\t"
        "v_fmac_f32 %[a2], %[w], v114\n\t"
        "v_fmac_f32 %[a3], %[w], v115\n\t"
        "ds_read_b128 v[112:115], %[o4] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v116\n\t"
        "v_fmac_f32 %[a1], %[w], v117\n\t"
        "v_fmac_f32 %[a2], %[w], v118\n\t"
        "v_fmac_f32 %[a3], %[w], v119\n\t"
        "ds_read_b128 v[116:119], %[o5] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v120\n\t"
        "v_fmac_f32 %[a1], %[w], v121\n\t"
        "v_fmac_f32 %[a2], %[w], v122\n\t"
        "v_fmac_f32 %[a3], %[w], v123\n\t"
        "ds_read_b128 v[120:123], %[o6] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v124\n\t"
        "v_fmac_f32 %[a1], %[w], v125\n\t"
        "v_fmac_f32 %[a2], %[w], v126\n\t"
        "v_fmac_f32 %[a3], %[w], v127\n\t"
        "ds_read_b128 v[124:127], %[o7] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v112\n\t"
        "v_fmac_f32 %[a1], %[w], v113\n\t"
        "v_fmac_f32 %[a2], %[w], v114\n\t"
        "v_fmac_f32 %[a3], %[w], v115\n\t"
        "ds_read_b128 v[112:115], %[o8] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v116\n\t"
        "v_fmac_f32 %[a1], %[w], v117\n\t"
        "v_fmac_f32 %[a2], %[w], v118\n\t"
        "v_fmac_f32 %[a3], %[w], v119\n\t"
        "ds_read_b128 v[116:119], %[o9] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v120\n\t"
        "v_fmac_f32 %[a1], %[w], v121\n\t"
        "v_fmac_f32 %[a2], %[w], v122\n\t"
        "v_fmac_f32 %[a3], %[w], v123\n\t"
        "ds_read_b128 v[120:123], %[o10] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v124\n\t"
        "v_fmac_f32 %[a1], %[w], v125\n\t"
        "v_fmac_f32 %[a2], %[w], v126\n\t"
        "v_fmac_f32 %[a3], %[w], v127\n\t"
        "ds_read_b128 v[124:127], %[o11] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v112\n\t"
        "v_fmac_f32 %[a1], %[w], v113\n\t"
        "v_fmac_f32 %[a2], %[w], v114\n\t"
        "v_fmac_f32 %[a3], %[w], v115\n\t"
        "ds_read_b128 v[112:115], %[o12] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v116\n\t"
        "v_fmac_f32 %[a1], %[w], v117\n\t"
        "v_fmac_f32 %[a2], %[w], v118\n\t"
        "v_fmac_f32 %[a3], %[w], v119\n\t"
        "ds_read_b128 v[116:119], %[o13] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v120\n\t"
        "v_fmac_f32 %[a1], %[w], v121\n\t"
        "v_fmac_f32 %[a2], %[w], v122\n\t"
        "v_fmac_f32 %[a3], %[w], v123\n\t"
        "ds_read_b128 v[120:123], %[o14] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v124\n\t"
        "v_fmac_f32 %[a1], %[w], v125\n\t"
        "v_fmac_f32 %[a2], %[w], v126\n\t"
        "v_fmac_f32 %[a3], %[w], v127\n\t"
        "ds_read_b128 v[124:127], %[o15] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v112\n\t"
        "v_fmac_f32 %[a1], %[w], v113\n\t"
        "v_fmac_f32 %[a2], %[w], v114\n\t"
        "v_fmac_f32 %[a3], %[w], v115\n\t"
        "s_waitcnt lgkmcnt(2)\n\t"
        "v_fmac_f32 %[a0], %[w], v116\n\t"
        "v_fmac_f32 %[a1], %[w], v117\n\t"
        "v_fmac_f32 %[a2], %[w], v118\n\t"
        "v_fmac_f32 %[a3], %[w], v119\n\t"
        "s_waitcnt lgkmcnt(1)\n\t"
        "v_fmac_f32 %[a0], %[w], v120\n\t"
        "v_fmac_f32 %[a1], %[w], v121\n\t"
        "v_fmac_f32 %[a2], %[w], v122\n\t"
        "v_fmac_f32 %[a3], %[w], v123\n\t"
        "s_waitcnt lgkmcnt(0)\n\t"
        "v_fmac_f32 %[a0], %[w], v124\n\t"
        "v_fmac_f32 %[a1], %[w], v125\n\t"
        "v_fmac_f32 %[a2], %[w], v126\n\t"
        "v_fmac_f32 %[a3], %[w], v127\n\t"
        : [a0] "+v"(acc[0]), [a1] "+v"(acc[1]), [a2] "+v"(acc[2]), [a3] "+v"(acc[3])
        : [o0] "v"(o[0]), [o1] "v"(o[1]), [o2] "v"(o[2]), [o3] "v"(o[3]), [o4] "v"(o[4]), [o5] "v"(o[5]), [o6] "v"(o[6]), [o7] "v"(o[7]), [o8] "v"(o[8]), [o9] "v"(o[9]), [o10] "v"(o[10]), [o11] "v"(o[11]), [o12] "v"(o[12]), [o13] "v"(o[13]), [o14] "v"(o[14]), [o15] "v"(o[15]),
          [w] "s"(w), [B] "n"(P * kBufSkew)
        : "v112", "v113", "v114", "v115", "v116", "v117", "v118", "v119", "v120", "v121", "v122", "v123",
          "v124", "v125", "v126", "v127", "memory");
}

// Eight connections, one scalar weight (see fma_block16s).
template <int P>
__device__ __forceinline__ void fma_block8s(float (&acc)[4], const uint32_t (&o)[8], float w) {
    asm volatile(
        "ds_read_b128 v[112:115], %[o0] offset:%[B]\n\t"
        "ds_read_b128 v[116:119], %[o1] offset:%[B]\n\t"
        "ds_read_b128 v[120:123], %[o2] offset:%[B]\n\t"
        "ds_read_b128 v[124:127], %[o3] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v112\n\t"
        "v_fmac_f32 %[a1], %[w], v113\n\t"
        "v_fmac_f32 %[a2], %[w], v114\n\t"
        "v_fmac_f32 %[a3], %[w], v115\n\t"
        "ds_read_b128 v[112:115], %[o4] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v116\n\t"
        "v_fmac_f32 %[a1], %[w], v117\n\t"
        "v_fmac_f32 %[a2], %[w], v118\n\t"
        "v_fmac_f32 %[a3], %[w], v119\n\t"
        "ds_read_b128 v[116:119], %[o5] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v120\n\t"
        "v_fmac_f32 %[a1], %[w], v121\n\t"
        "v_fmac_f32 %[a2], %[w], v122\n\t"
        "v_fmac_f32 %[a3], %[w], v123\n\t"
        "ds_read_b128 v[120:123], %[o6] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v124\n\t"
        "v_fmac_f32 %[a1], %[w], v125\n\t"
        "v_fmac_f32 %[a2], %[w], v126\n\t"
        "v_fmac_f32 %[a3], %[w], v127\n\t"
        "ds_read_b128 v[124:127], %[o7] offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v112\n\t"
        "v_fmac_f32 %[a1], %[w], v113\n\t"
        "v_fmac_f32 %[a2], %[w], v114\n\t"
        "v_fmac_f32 %[a3], %[w], v115\n\t"
        "s_waitcnt lgkmcnt(2)\n\t"
        "v_fmac_f32 %[a0], %[w], v116\n\t"
        "v_fmac_f32 %[a1], %[w], v117\n\t"
        "v_fmac_f32 %[a2], %[w], v118\n\t"
        "v_fmac_f32 %[a3], %[w], v119\n\t"
        "s_waitcnt lgkmcnt(1)\n\t"
        "v_fmac_f32 %[a0], %[w], v120\n\t"
        "v_fmac_f32 %[a1], %[w], v121\n\t"
        "v_fmac_f32 %[a2], %[w], v122\n\t"
        "v_fmac_f32 %[a3], %[w], v123\n\t"
        "s_waitcnt lgkmcnt(0)\n\t"
        "v_fmac_f32 %[a0], %[w], v124\n\t"
        "v_fmac_f32 %[a1], %[w], v125\n\t"
        "v_fmac_f32 %[a2], %[w], v126\n\t"
        "v_fmac_f32 %[a3], %[w], v127\n\t"
        : [a0] "+v"(acc[0]), [a1] "+v"(acc[1]), [a2] "+v"(acc[2]), [a3] "+v"(acc[3])
        : [o0] "v"(o[0]), [o1] "v"(o[1]), [o2] "v"(o[2]), [o3] "v"(o[3]), [o4] "v"(o[4]), [o5] "v"(o[5]), [o6] "v"(o[6]), [o7] "v"(o[7]),
          [w] "s"(w), [B] "n"(P * kBufSkew)
        : "v112", "v113", "v114", "v115", "v116", "v117", "v118", "v119", "v120", "v121", "v122", "v123",
          "v124", "v125", "v126", "v127", "memory");
}

// Eight connections whose LDS addresses are packed two per register as (byte address >> 4)
// in 16 bits each, one scalar weight.  An SDWA shift turns a half into the byte address,
// written into the first register of the read's own destination.  sh4 (scalar) holds 4.  Two reads
// in flight (with 16 waves per CU the LDS stays busy at this depth, and the kernel that
// uses this block needs the registers).
template <int P>
__device__ __forceinline__ void fma_block8ps(float (&acc)[4], uint32_t p0, uint32_t p1, uint32_t p2, uint32_t p3,
                                             float w, uint32_t sh4) {
    asm volatile(
        "v_lshlrev_b32_sdwa v120, %[s4], %[p0] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
        "ds_read_b128 v[120:123], v120 offset:%[B]\n\t"
        "v_lshlrev_b32_sdwa v124, %[s4], %[p0] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n\t"
        "ds_read_b128 v[124:127], v124 offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(1)\n\t"
        "v_fmac_f32 %[a0], %[w], v120\n\t"
        "v_fmac_f32 %[a1], %[w], v121\n\t"
        "v_fmac_f32 %[a2], %[w], v122\n\t"
        "v_fmac_f32 %[a3], %[w], v123\n\t"
        "v_lshlrev_b32_sdwa v120, %[s4], %[p1] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
        "ds_read_b128 v[120:123], v120 offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(1)\n\t"
        "v_fmac_f32 %[a0], %[w], v124\n\t"
        "v_fmac_f32 %[a1], %[w], v125\n\t"
        "v_fmac_f32 %[a2], %[w], v126\n\t"
        "v_fmac_f32 %[a3], %[w], v127\n\t"
        "v_lshlrev_b32_sdwa v124, %[s4], %[p1] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n\t"
        "ds_read_b128 v[124:127], v124 offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(1)\n\t"
        "v_fmac_f32 %[a0], %[w], v120\n\t"
        "v_fmac_f32 %[a1], %[w], v121\n\t"
        "v_fmac_f32 %[a2], %[w], v122\n\t"
        "v_fmac_f32 %[a3], %[w], v123\n\t"
        "v_lshlrev_b32_sdwa v120, %[s4], %[p2] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
        "ds_read_b128 v[120:123], v120 offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(1)\n\t"
        "v_fmac_f32 %[a0], %[w], v124\n\t"
        "v_fmac_f32 %[a1], %[w], v125\n\t"
        "v_fmac_f32 %[a2], %[w], v126\n\t"
        "v_fmac_f32 %[a3], %[w], v127\n\t"
        "v_lshlrev_b32_sdwa v124, %[s4], %[p2] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n\t"
        "ds_read_b128 v[124:127], v124 offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(1)\n\t"
        "v_fmac_f32 %[a0], %[w], v120\n\t"
        "v_fmac_f32 %[a1], %[w], v121\n\t"
        "v_fmac_f32 %[a2], %[w], v122\n\t"
        "v_fmac_f32 %[a3], %[w], v123\n\t"
        "v_lshlrev_b32_sdwa v120, %[s4], %[p3] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
        "ds_read_b128 v[120:123], v120 offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(1)\n\t"
        "v_fmac_f32 %[a0], %[w], v124\n\t"
        "v_fmac_f32 %[a1], %[w], v125\n\t"
        "v_fmac_f32 %[a2], %[w], v126\n\t"
        "v_fmac_f32 %[a3], %[w], v127\n\t"
        "v_lshlrev_b32_sdwa v124, %[s4], %[p3] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n\t"
        "ds_read_b128 v[124:127], v124 offset:%[B]\n\t"
        "s_waitcnt lgkmcnt(1)\n\t"
        "v_fmac_f32 %[a0], %[w], v120\n\t"
        "v_fmac_f32 %[a1], %[w], v121\n\t"
        "v_fmac_f32 %[a2], %[w], v122\n\t"
        "v_fmac_f32 %[a3], %[w], v123\n\t"
        "s_waitcnt lgkmcnt(0)\n\t"
        "v_fmac_f32 %[a0], %[w], v124\n\t"
        "v_fmac_f32 %[a1], %[w], v125\n\t"
        "v_fmac_f32 %[a2], %[w], v126\n\t"
        "v_fmac_f32 %[a3], %[w], v127\n\t"
        : [a0] "+v"(acc[0]), [a1] "+v"(acc[1]), [a2] "+v"(acc[2]), [a3] "+v"(acc[3])
        : [p0] "v"(p0), [p1] "v"(p1), [p2] "v"(p2), [p3] "v"(p3), [w] "s"(w), [s4] "s"(sh4), [B] "n"(P * kBufSkew)
        : "v120", "v121", "v122", "v123", "v124", "v125", "v126", "v127", "memory");
}

// Maximum / minimum over each row of 16 lanes, left in all 16 of them: four DPP rotations inside the row.
__device__ __forceinline__ int row16_max(int v) {
    v = max(v, __builtin_amdgcn_mov_dpp(v, 0x128, 0xF, 0xF, true));  // row_ror:8
    v = max(v, __builtin_amdgcn_mov_dpp(v, 0x124, 0xF, 0xF, true));  // row_ror:4
    v = max(v, __builtin_amdgcn_mov_dpp(v, 0x122, 0xF, 0xF, true));  // row_ror:2
    v = max(v, __builtin_amdgcn_mov_dpp(v, 0x121, 0xF, 0xF, true));  // row_ror:1
    return v;
}
__device__ __forceinline__ int row16_min(int v) {
    v = min(v, __builtin_amdgcn_mov_dpp(v, 0x128, 0xF, 0xF, true));
    v = min(v, __builtin_amdgcn_mov_dpp(v, 0x124, 0xF, 0xF, true));
    v = min(v, __builtin_amdgcn_mov_dpp(v, 0x122, 0xF, 0xF, true));
    v = min(v, __builtin_amdgcn_mov_dpp(v, 0x121, 0xF, 0xF, true));
    return v;
}

// Number of set bytes among flags[0 .. n), counted by the whole workgroup.  red: 17 ints of LDS.
// Four 16-byte loads per thread are in flight at a time (the count sits on every workgroup's way in).
__device__ __forceinline__ int count_flags(const uint8_t* __restrict__ flags, int n, int* red) {
    const int tid = threadIdx.x;
    int c = 0;
    for (int i0 = tid * 16; i0 < n; i0 += 4 * kBlk * 16) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = i0 + u * kBlk * 16;
            v[u] = make_uint4(0u, 0u, 0u, 0u);
            if (i + 16 <= n) v[u] = *reinterpret_cast<const uint4*>(flags + i);
            else
                for (int k = i; k < n; ++k) c += flags[k];  // the ragged end: one thread, at most 15 bytes
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)  // bytes are 0 or 1: the population count of a word is its number of flags
            c += __popc(v[u].x) + __popc(v[u].y) + __popc(v[u].z) + __popc(v[u].w);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) c += __shfl_xor(c, d, 64);
    __syncthreads();  // red may still be read from a call before
    if ((tid & 63) == 0) red[tid >> 6] = c;
    __syncthreads();
    int t = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) t += red[w];
    return t;
}

// How a layer's kernel gets its list of active rows (a2, the host loop of Listing 1 between two layers,
// folded into the layer that needs its result, so that a layer is one launch).  The previous layer
// left one flag byte per row it wrote ("has a positive output"); every workgroup counts them for
// itself, works out which row groups of the compacted list are its own, and writes that slice of the
// list -- the slots of its rows in the buffer the previous layer wrote, and their original row numbers
// -- before it reads it back.  Workgroups with the same rows (other column blocks) write the same
// values to the same places; nothing a workgroup reads was written by another workgroup of the launch.
struct RowLists {
    const uint8_t* flags_prev;  // [*count_prev] flags of the rows the previous layer wrote; NULL: the lists below are
                                // complete already (later passes of a layer of several passes)
    const int* count_prev;      // rows the previous layer wrote
    const int* gid_prev;        // [*count_prev] their original row numbers
    int* cat;                   // out: slot (in the previous layer's buffer) of the i-th active row; not written when
                                // no row died (then it is i)
    int* gid;                   // out: its original row number
    int* count;                 // out (workgroup 0): number of active rows A
    int* host_count;            // out (workgroup 0): the same, in pinned host memory
    uint8_t* flags_clear;       // the buffer the next layer will raise its flags in: this layer clears its rows of it
};

// Entries of the list are read from the same address by every lane, but from memory the kernel itself
// wrote a moment ago, so they arrive in vector registers: back to scalar ones (row bases are scalar
// operands of the tile loads).
__device__ __forceinline__ int4 uniform4(int4 v) {
    return make_int4(__builtin_amdgcn_readfirstlane(v.x), __builtin_amdgcn_readfirstlane(v.y),
                     __builtin_amdgcn_readfirstlane(v.z), __builtin_amdgcn_readfirstlane(v.w));
}
__device__ __forceinline__ int2 uniform2(int2 v) {
    return make_int2(__builtin_amdgcn_readfirstlane(v.x), __builtin_amdgcn_readfirstlane(v.y));
}

// 64 consecutive entries of the workgroup's slice of the list, entry k in lane k of one register; a tile's
// entries are picked out with v_readlane.  The tile loop therefore meets a load from the list, and the
// wait for it (which also waits for every tile load in flight), once per 64 entries, not once per tile.
// Entries past the slice's end repeat its last entry: a valid row to re-read, for the ragged last group.
struct ListWindow {
    const int* cat;
    int first, end;  // the slice [first, end) of the list, end > first
    int lo;          // entries [lo, lo + 64) are held
    int v;
    bool identity;   // the list is 0, 1, 2, ...: nothing is read
    __device__ __forceinline__ ListWindow(const int* cat_, int first_, int end_, bool identity_)
        : cat(cat_), first(first_), end(end_), lo(first_), identity(identity_) {
        fill();
    }
    __device__ __forceinline__ void fill() {
        const int e = min(lo + (int)(threadIdx.x & 63), end - 1);
        v = identity ? e : cat[e];
    }
    __device__ __forceinline__ void seek(int e) {  // e: the same in every lane
        const int want = first + ((e - first) & ~63);
        if (want != lo) {
            lo = want;
            fill();
        }
    }
    __device__ __forceinline__ int4 get4(int e) {  // entries e .. e+3, e - first a multiple of 4
        seek(e);
        const int k = e - lo;
        return make_int4(__builtin_amdgcn_readlane(v, k), __builtin_amdgcn_readlane(v, k + 1),
                         __builtin_amdgcn_readlane(v, k + 2), __builtin_amdgcn_readlane(v, k + 3));
    }
    __device__ __forceinline__ int2 get2(int e) {
        seek(e);
        const int k = e - lo;
        return make_int2(__builtin_amdgcn_readlane(v, k), __builtin_amdgcn_readlane(v, k + 1));
    }
    __device__ __forceinline__ int last() const { return identity ? end - 1 : __builtin_amdgcn_readfirstlane(cat[end - 1]); }
};

// Workgroup -> (column block, row groups): a launch has ncb column blocks times Q chunks of row groups, the G
// column blocks that read the same rows get workgroup ids that are equal modulo 8 (one XCD, one L2).  The
// lists are derived on the way.  red: 17 ints, scan: 17 ints of LDS.
struct WorkItem {
    int cb, A, g0, g1;
    bool identity;  // no row died in the previous layer: entry i of the list is i, and the list was not written
};
__device__ __forceinline__ bool derive_work(const RowLists& rl, int ncb, int G, int Q, WorkItem& w, int rows_per_group,
                                            int* red, int* scan) {
    const int tid = threadIdx.x;
    const int xcd = blockIdx.x & 7;
    const int slot = blockIdx.x >> 3;
    const int unit = (slot / G) * 8 + xcd;
    const int sub = slot - (slot / G) * G;
    const int ngrp = ncb / G;
    const bool has_unit = unit < ngrp * Q;
    if (!has_unit && blockIdx.x != 0) return false;
    if (!rl.flags_prev) {  // lists and count are in place
        if (!has_unit) return false;
        const int q = unit / ngrp;
        w.cb = (unit - q * ngrp) * G + sub;
        w.A = __builtin_amdgcn_readfirstlane(*rl.count);
        const int ngroups = (w.A + rows_per_group - 1) / rows_per_group;
        const int per = (ngroups + Q - 1) / Q;
        w.g0 = q * per;
        w.g1 = min(ngroups, w.g0 + per);
        w.identity = w.A == __builtin_amdgcn_readfirstlane(*rl.count_prev);  // as the layer's first pass found it
        return w.g0 < w.g1;
    }
    // the same in every lane: said out loud, so that everything derived from them stays in scalar registers
    const int Aprev = __builtin_amdgcn_readfirstlane(*rl.count_prev);
    const int A = __builtin_amdgcn_readfirstlane(count_flags(rl.flags_prev, Aprev, red));
    if (blockIdx.x == 0 && tid == 0) {
        *rl.count = A;
        // the host reads nothing else that this kernel writes before the stream is drained: no release (which
        // would write back the L2), just a store that goes through to host memory
        __hip_atomic_store(rl.host_count, A, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
    }
    if (!has_unit) return false;
    const int q = unit / ngrp;
    w.cb = (unit - q * ngrp) * G + sub;
    w.A = A;
    const int ngroups = (A + rows_per_group - 1) / rows_per_group;
    const int per = (ngroups + Q - 1) / Q;
    w.g0 = q * per;
    w.g1 = min(ngroups, w.g0 + per);
    if (w.g0 >= w.g1) return false;
    // my slice of the list: ranks [r0, r1) among the set flags (the list's last entry too, which the ragged
    // last group re-reads: it is in the last slice, and only the workgroups of that slice use it)
    const int r0 = w.g0 * rows_per_group;
    const int r1 = min(A, w.g1 * rows_per_group);
    for (int r = r0 + tid; r < r1; r += kBlk) rl.flags_clear[r] = 0;
    w.identity = A == Aprev;
    if (w.identity) {  // nobody died: the slots are 0, 1, 2, ... (not written: ListWindow counts them up itself)
        for (int r = r0 + tid; r < r1; r += kBlk) rl.gid[r] = rl.gid_prev[r];
    } else {
        // walk the flags in chunks of 16 per thread; an exclusive scan over the workgroup's counts gives the ranks
        const int lane = tid & 63, wave = tid >> 6;
        int base = 0;  // set flags before the chunk
        for (int c0 = 0; c0 < Aprev && base < r1; c0 += kBlk * 16) {
            const int i = c0 + tid * 16;
            uint32_t f[4] = {0, 0, 0, 0};
            if (i + 16 <= Aprev) {
                const uint4 v = *reinterpret_cast<const uint4*>(rl.flags_prev + i);
                f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
            } else {
                for (int k = i; k < Aprev; ++k) f[(k - i) >> 2] |= (uint32_t)rl.flags_prev[k] << (8 * ((k - i) & 3));
            }
            const int mine = __popc(f[0]) + __popc(f[1]) + __popc(f[2]) + __popc(f[3]);
            int incl = mine;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int up = __shfl_up(incl, d, 64);
                if (lane >= d) incl += up;
            }
            __syncthreads();  // scan[] may still be read from the chunk before
            if (lane == 63) scan[wave] = incl;
            __syncthreads();
            if (tid == 0) {
                int run = 0;
                for (int k = 0; k < 16; ++k) {
                    const int t = scan[k];
                    scan[k] = run;
                    run += t;
                }
                scan[16] = run;
            }
            __syncthreads();
            int rank = base + scan[wave] + incl - mine;
            if (mine && rank < r1 && rank + mine > r0) {
#pragma unroll
                for (int k = 0; k < 16; ++k)
                    if ((f[k >> 2] >> (8 * (k & 3))) & 1u) {
                        if (rank >= r0 && rank < r1) {
                            rl.cat[rank] = i + k;
                            rl.gid[rank] = rl.gid_prev[i + k];
                        }
                        ++rank;
                    }
            }
            base += scan[16];
        }
    }
    if (!w.identity) __syncthreads();  // the slice is written (workgroup-scope release / acquire): it may be read now
    return true;
}

// Tile staging shared by the fused kernels.  A lane owns 4 neighbouring columns of the
// tile: stage_load fetches them from the tile's 4 rows (16 bytes per row; rows past the
// last active one re-read the last active row and are never stored), stage_store
// transposes the 4x4 block in registers and writes one 16-byte entry (the 4 rows of a
// column) per column.  addr = LDS address of the lane's store group in the buffer to
// fill; qp = bank quad (times 16) of each of the 4 columns inside its group's 256-byte
// row, one per byte (0 for layouts where the address already says it all).
__device__ __forceinline__ void stage_load(f32x4 (&st)[kRows], const float* __restrict__ Yin, int N, int4 c4,
                                           int row0, int A, int cat_last, size_t coff) {
    st[0] = *reinterpret_cast<const f32x4*>(Yin + (size_t)c4.x * N + coff);
    st[1] = *reinterpret_cast<const f32x4*>(Yin + (size_t)(row0 + 1 < A ? c4.y : cat_last) * N + coff);
    st[2] = *reinterpret_cast<const f32x4*>(Yin + (size_t)(row0 + 2 < A ? c4.z : cat_last) * N + coff);
    st[3] = *reinterpret_cast<const f32x4*>(Yin + (size_t)(row0 + 3 < A ? c4.w : cat_last) * N + coff);
}
__device__ __forceinline__ void stage_store(f32x4 (&st)[kRows], uint32_t addr, uint32_t qp) {
    using lds_f4 = __attribute__((address_space(3))) f32x4;
    // The loads of this tile were issued a step ago.  Pin the point where their results are
    // first touched, otherwise the register shuffles of the transpose are scheduled right
    // behind the loads and every load turns synchronous.
    asm volatile("" : "+v"(st[0]), "+v"(st[1]), "+v"(st[2]), "+v"(st[3]));
    *reinterpret_cast<lds_f4*>(addr + (qp & 0xffu) + 0 * 512) = f32x4{st[0].x, st[1].x, st[2].x, st[3].x};
    *reinterpret_cast<lds_f4*>(addr + ((qp >> 8) & 0xffu) + 1 * 512) = f32x4{st[0].y, st[1].y, st[2].y, st[3].y};
    *reinterpret_cast<lds_f4*>(addr + ((qp >> 16) & 0xffu) + 2 * 512) = f32x4{st[0].z, st[1].z, st[2].z, st[3].z};
    *reinterpret_cast<lds_f4*>(addr + (qp >> 24) + 3 * 512) = f32x4{st[0].w, st[1].w, st[2].w, st[3].w};
}

// 4x4 transpose inside each lane quartet: lane 4q+i comes in with four values of its own (y0..y3 = rows 0..3 of
// neuron 4q+i) and leaves with y_k = what lane 4q+k held in its y_i (row i of neurons 4q..4q+3).  Two exchanges,
// with the neighbour two lanes away and then the one next door, each a select whose one operand comes in through
// DPP: eight instructions.  (As selects and DPP moves written in C++ they were sixteen.)
__device__ __forceinline__ void transpose_quartet(float& y0, float& y1, float& y2, float& y3) {
    float n0, n1, n2, n3, m0, m1, m2, m3;
    const uint64_t hi2 = 0xCCCCCCCCCCCCCCCCull;  // lanes with bit 1 set
    const uint64_t hi1 = 0xAAAAAAAAAAAAAAAAull;  // lanes with bit 0 set
    asm volatile(
        "s_nop 1\n\t"  // the values may have been written by the instruction before; DPP reads need two wait states
        "s_not_b64 vcc, %[hi2]\n\t"
        "v_cndmask_b32_dpp %[n0], %[y2], %[y0], vcc quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_cndmask_b32_dpp %[n1], %[y3], %[y1], vcc quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_mov_b64 vcc, %[hi2]\n\t"
        "v_cndmask_b32_dpp %[n2], %[y0], %[y2], vcc quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "v_cndmask_b32_dpp %[n3], %[y1], %[y3], vcc quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
        "s_not_b64 vcc, %[hi1]\n\t"
        "v_cndmask_b32_dpp %[m0], %[n1], %[n0], vcc quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_nop 0\n\t"
        "v_cndmask_b32_dpp %[m2], %[n3], %[n2], vcc quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "s_mov_b64 vcc, %[hi1]\n\t"
        "v_cndmask_b32_dpp %[m1], %[n0], %[n1], vcc quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        "v_cndmask_b32_dpp %[m3], %[n2], %[n3], vcc quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
        : [n0] "=&v"(n0), [n1] "=&v"(n1), [n2] "=&v"(n2), [n3] "=&v"(n3), [m0] "=&v"(m0), [m1] "=&v"(m1),
          [m2] "=&v"(m2), [m3] "=&v"(m3)
        : [y0] "v"(y0), [y1] "v"(y1), [y2] "v"(y2), [y3] "v"(y3), [hi2] "s"(hi2), [hi1] "s"(hi1)
        : "vcc", "scc");
    y0 = m0;
    y1 = m1;
    y2 = m2;
    y3 = m3;
}

// Epilogue of one 4-row group of one neuron (Eq. 1: bias, ReLU, clip at 32): lane 4q+i
// holds rows 0..3 of neuron 4q+i; a 4x4 transpose inside each lane quartet (two DPP
// exchanges) leaves it with row i of neurons 4q..4q+3, which is one 16-byte store.
// Clears the accumulators.  Returns bit r set if row r has a positive output anywhere in
// the wave (lanes past the last neuron carry zero weights and zero bias, so their y is 0).
// The output goes out with the non-temporal hint: a layer's output is read again only by the next layer, by when
// (at the sizes that matter) it has long left the caches, and without the hint it pushes out the input tiles that
// workgroups share.  Measured: 1.5 to 3 % per layer on outputs of 0.25 GB and more, nothing either way on small
// ones (1.6 % lost on one of 0.13 GB).
__device__ __forceinline__ unsigned finish_rows(float (&a)[kRows], float bj, float* __restrict__ Yout, int N, int j,
                                                bool jok, int row0, int nlive, int lane) {
    float y0 = fminf(fmaxf(a[0] + bj, 0.0f), kClip);
    float y1 = fminf(fmaxf(a[1] + bj, 0.0f), kClip);
    float y2 = fminf(fmaxf(a[2] + bj, 0.0f), kClip);
    float y3 = fminf(fmaxf(a[3] + bj, 0.0f), kClip);
    a[0] = a[1] = a[2] = a[3] = 0.0f;
    const unsigned pos = (__builtin_amdgcn_ballot_w64(y0 > 0.0f) != 0ull ? 1u : 0u) |
                         (__builtin_amdgcn_ballot_w64(y1 > 0.0f) != 0ull ? 2u : 0u) |
                         (__builtin_amdgcn_ballot_w64(y2 > 0.0f) != 0ull ? 4u : 0u) |
                         (__builtin_amdgcn_ballot_w64(y3 > 0.0f) != 0ull ? 8u : 0u);
    transpose_quartet(y0, y1, y2, y3);
    const int r = lane & 3;
    if (jok && r < nlive)
        __builtin_nontemporal_store(f32x4{y0, y1, y2, y3}, reinterpret_cast<f32x4*>(Yout + (size_t)(row0 + r) * N + (j & ~3)));
    return pos;
}

// A layer whose neurons have more than 32 connections (general layers, Section II-A-1) runs with several
// lanes per neuron: a neuron of K connections is cut into ceil(K/32) parts of up to 32, each part is one lane's
// work, and a workgroup takes a run of neighbouring neurons (a multiple of 4, at most 1024) that have at most 1024
// parts together.  Inside a workgroup the parts are given to the lanes in the order of their lengths, longest
// first, so that a wave's 64 lanes have about equally many connections and a wave runs only the blocks of 8
// steps its longest lane needs -- the zero padding of Section III-A-3 at the granularity of a wave.  After the
// last step of a row group every lane leaves its four sums (one per row of the tile) in its slot of a 16-KB LDS
// array -- a neuron's parts have neighbouring slots -- and at the start of the next step, behind the step's
// barrier, the workgroup's LAST lanes (the ones with the shortest parts) add up the slots of its neurons in part
// order, one neuron per lane, add the bias, clip and store (finish_rows) while the other waves are at the next
// tile's arithmetic; two sets of slots alternate.  No partial sum leaves the CU.
struct VirtInfo {
    const uint16_t* slot;  // [nblk][kBlk] the lane's slot
    const uint8_t* nb8;    // [nblk][16] blocks of 8 steps wave w of the workgroup runs (0..4)
    const int2* range;     // [nblk] {first neuron, number of neurons} of the workgroup; {N, 0}: none
    const uint32_t* fin;   // [nblk][kBlk] entry i < number of neurons: first slot | number of slots << 16 of the workgroup's i-th neuron
    uint32_t part_off;     // byte offset of the two sets of slots inside the dynamic LDS (behind the tile pair)
};

// ---------------------------------------------------------------------------
// a1: fused SpMM + bias + clipped ReLU for one layer (Eq. 1), plus the per-row
// "has a positive output" flag that Listings 1 and 2 keep in active[].
//
// Yin is read through the list of active rows that the kernel derives first (RowLists:
// slot of every active row in the buffer written by the previous layer); row i of the
// list is written to slot i of Yout.  A launch has ncb column blocks (output blocks, or
// units of 2048 / 4096 neurons) times Q row chunks; consecutive workgroup ids go to
// consecutive XCDs (8 of them, each with its own L2), and the G column blocks that read
// the same rows through overlapping windows get ids that are equal modulo 8, so they
// share one L2.  A workgroup handles row groups [q*per, (q+1)*per) of ceil(A/4).
//
// VIRT: several lanes per neuron (VirtInfo); the launch computes the outputs of its workgroups' neurons.
// ---------------------------------------------------------------------------
template <bool MULTI, bool VIRT = false>
__global__ __launch_bounds__(kBlk) void fused_layer_kernel(
    const float* __restrict__ Yin, float* __restrict__ Yout, uint8_t* __restrict__ flags,
    RowLists rl, LayerWeights w,
    const float* __restrict__ bias, int N, int nblk, int G, int Q, VirtInfo vi = VirtInfo{}) {
    extern __shared__ float4 lds4[];
    const int tid = threadIdx.x;

    WorkItem wi;  // my output block and row groups
    int *rl_red, *rl_scan;
    if constexpr (VIRT) {  // every byte of LDS is spoken for (two tiles, two sets of slots): borrow the first tile
        rl_red = reinterpret_cast<int*>(lds4);
        rl_scan = rl_red + 32;
    } else {
        __shared__ int red_mem[17], scan_mem[17];
        rl_red = red_mem;
        rl_scan = scan_mem;
    }
    if (!derive_work(rl, nblk, G, Q, wi, kRows, rl_red, rl_scan)) return;
    if (VIRT) __syncthreads();  // ... and give it back only when every wave is done with it
    const int* cat = rl.cat;      // my slice of it was written just now
    const int b = wi.cb, A = wi.A, g0 = wi.g0, g1 = wi.g1;
    const int2 mine = VIRT ? vi.range[b] : make_int2(b * kBlk, kBlk);  // my workgroup's neurons
    if (VIRT && mine.y == 0) return;  // a workgroup past the last neuron

    // The neuron whose result this lane finishes and stores.  VIRT: the workgroup's last mine.y lanes finish its
    // neurons -- the lanes with the shortest parts, whose waves have time to spare.
    const int fl = tid - (kBlk - mine.y);  // which of my workgroup's neurons
    const int j = mine.x + fl;
    const bool jok = j < N && fl >= 0;
    const int2 win = w.win[b];
    const int c_lo = win.x;
    const int ncols = win.y;
    const int nstage = MULTI ? (ncols + kCap - 1) / kCap : 1;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds4;  // LDS byte address of the tile pair

    // Connections of my output neuron, in registers for the whole kernel.
    // off = LDS byte address (buffer 0) of the column inside its stage; MULTI also
    // keeps the stage numbers, eight 4-bit fields per register.
    uint32_t off[kNnz];
    float wv[kNnz];
    uint32_t stg[MULTI ? kNnz / 8 : 1] = {};
    {
        const uint16_t* prel = w.rel + (size_t)b * kNnz * kBlk + tid;
        const float* pval = w.val + (size_t)b * kNnz * kBlk + tid;
#pragma unroll
        for (int k = 0; k < kNnz; ++k) {
            const uint32_t rel = prel[k * kBlk];
            wv[k] = pval[k * kBlk];
            off[k] = lds_base + tile_offset(rel & (kCap - 1));
            if (MULTI) stg[k >> 3] |= (rel >> kCapLog2) << (4 * (k & 7));
        }
    }
    if (MULTI) {
        // A connection that belongs to another stage reads its slot of the current tile all
        // the same and contributes with weight 0.  That is exact as long as whatever lies in
        // the slot is finite, so the tile pair starts out as zeros (later contents are
        // activations; slots past a narrow last stage keep older ones).
        using lds_f4 = __attribute__((address_space(3))) f32x4;
        for (uint32_t o = 16u * tid; o < tile_pair_bytes(kCap); o += 16u * kBlk)
            *reinterpret_cast<lds_f4*>(lds_base + o) = f32x4{0.f, 0.f, 0.f, 0.f};
        __syncthreads();
    }
    const float bj = jok ? bias[j] : 0.0f;
    // VIRT: where my sums go, and how many blocks of 8 steps my wave runs
    const uint32_t part_base = lds_base + (VIRT ? vi.part_off : 0u);
    const uint32_t part_addr = part_base + 16u * (VIRT ? (uint32_t)vi.slot[(size_t)b * kBlk + tid] : 0u);
    const int nb = VIRT ? __builtin_amdgcn_readfirstlane((int)vi.nb8[b * 16 + (tid >> 6)]) : kNnz / 8;
    const uint32_t fin = (VIRT && fl >= 0) ? vi.fin[(size_t)b * kBlk + fl] : 0u;  // my neuron's slots
    int pending = -1;  // VIRT: the row group whose sums wait in the slots to be finished

    const int T = (g1 - g0) * nstage;  // pipeline steps: (row group, stage) pairs
    // Staging: lane t owns columns 4t..4t+3 of the stage: one 16-byte load per row,
    // a 4x4 transpose in registers, four 16-byte LDS stores (entry = the 4 rows of
    // one column).  Waves whose columns lie past the stage's last column skip the
    // work; inside the last wave, lanes past it re-read the last 4 columns.
    f32x4 st[kRows];
    const int wave_col = (tid & ~63) * 4;  // first column of my wave
    // LDS address of column 4t + a is st_addr + a*512 + st_quad[a].  Single-stage layers
    // use the balanced layout (the quads come from the set-up), the others col_slot().
    uint32_t st_addr = lds_base + tile_offset(col_slot(4 * tid));
    uint32_t qp = 0;  // byte a = quad of column 4t + a, times 16
    if (!MULTI) {
        st_addr = lds_base + tile_offset(store_group(4 * tid) << 4);
        qp = w.qsel[(size_t)b * kBlk + tid];
    }
    ListWindow rows_of(cat, g0 * kRows, min(A, g1 * kRows), wi.identity);
    const int cat_last = rows_of.last();  // used by the last, ragged group only: then the list's last entry
    int4 c4 = make_int4(0, 0, 0, 0);  // slots (in Yin) of the 4 rows of the tile to load next

    // the four rows of the tile to load next (the last, ragged group repeats the list's last row)
    auto fetch_rows = [&](int t) {
        const int gi = MULTI ? t / nstage : t;
        c4 = rows_of.get4((g0 + gi) * kRows);
    };
    auto load_tile = [&](int t) {
        const int gi = MULTI ? t / nstage : t;
        const int s = MULTI ? t - gi * nstage : 0;
        const int left = ncols - s * kCap;  // columns in this stage (a multiple of 4, may exceed kCap)
        if (wave_col >= left) return;
        const int row0 = (g0 + gi) * kRows;
        const size_t coff = (size_t)win_col(c_lo, s * kCap + min(4 * tid, left - 4), N);  // windows are cyclic
        stage_load(st, Yin, N, c4, row0, A, cat_last, coff);
    };
    auto store_tile = [&](int P, int t) {
        const int gi = MULTI ? t / nstage : t;
        const int s = MULTI ? t - gi * nstage : 0;
        const int left = ncols - s * kCap;
        if (wave_col >= left) return;
        // the four store addresses are worked out per tile from two registers, not kept in four across the loop
        uint32_t q = qp, a = st_addr;
        if (!MULTI) asm volatile("" : "+v"(q), "+v"(a));
        stage_store(st, a + P * kBufSkew, q);
    };

    float acc[kRows] = {0.f, 0.f, 0.f, 0.f};
    // The four waves that share a SIMD get different issue priorities (first wave
    // highest).  Without it all 16 waves hit the LDS in lock step after each barrier
    // and the last one served reaches the next barrier ~2000 cycles after the first;
    // measured gain on the 65536-neuron layers: 3-4 %.
    {
        const int pw = __builtin_amdgcn_readfirstlane(3 - ((threadIdx.x >> 8) & 3));
        if (pw == 1) __builtin_amdgcn_s_setprio(1);
        else if (pw == 2) __builtin_amdgcn_s_setprio(2);
        else if (pw == 3) __builtin_amdgcn_s_setprio(3);
    }

    // connections kbeg .. kbeg+15 of the tile in buffer P
    auto compute = [&](auto Ptag, int s, auto Ktag) {
        constexpr int P = decltype(Ptag)::value;
        constexpr int kbeg = decltype(Ktag)::value;
#pragma unroll
        for (int kk = 0; kk < 16; kk += 8) {
            const int k0 = kbeg + kk;
            uint32_t o[8];
            float v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                o[i] = off[k0 + i];
                v[i] = wv[k0 + i];
                if (MULTI) {
                    // field k of stg is compared through a word that changes with s, so that the
                    // 32 extracted stage numbers are not kept in registers across the loop
                    const int k = k0 + i;
                    const uint32_t x = stg[k >> 3] ^ ((uint32_t)s * 0x11111111u);
                    v[i] = (x & (15u << (4 * (k & 7)))) == 0u ? v[i] : 0.0f;
                }
            }
            if (!VIRT || (k0 >> 3) < nb) fma_block8<P>(acc, o, v);  // VIRT: the blocks my wave's longest lane needs
            // keep each block's masked weights next to their block: hoisted, they would
            // need 32 more registers
            if (MULTI) __builtin_amdgcn_sched_barrier(0);
        }
    };

    const int lane = tid & 63;
    // Exchange between lanes l and l^1 / l^2 of a quartet (DPP quad permutes).
    auto epilogue = [&](int g) {
        const int row0 = g * kRows;
        const int nlive = min(kRows, A - row0);  // rows of this group that exist (>= 1)
        if (VIRT) {
            // My part's four sums go to my slot, in the set of slots of this group's parity.  They are added up at
            // the start of the next step (finish_pending), behind this step's barrier and under the other waves'
            // arithmetic; the set is written again two groups later, with a barrier in between.
            using lds_f4 = __attribute__((address_space(3))) f32x4;
            *reinterpret_cast<lds_f4*>(part_addr + (uint32_t)(g & 1) * (16u * kBlk)) = f32x4{acc[0], acc[1], acc[2], acc[3]};
            acc[0] = acc[1] = acc[2] = acc[3] = 0.0f;
            pending = g;
            return;
        }
        const unsigned pos = finish_rows(acc, bj, Yout, N, j, jok, row0, nlive, lane);
        if (lane < nlive && ((pos >> lane) & 1u)) flags[row0 + lane] = 1;  // lane r raises row r's flag
    };

    // One pipeline step with compile-time buffer index P.  On entry tile t is in
    // buffer P and the registers st hold tile t+1 (or its loads are in flight).
    // Half way through, tile t+1 goes to the other buffer -- nobody reads that one
    // before the barrier below -- and the loads of tile t+2 are issued, so they have
    // a whole step to land and the barrier never waits for global memory.
    // VIRT: the neuron's lane adds up its parts' sums in part order, then bias, clip and store as everywhere
    auto finish_pending = [&]() {
        if (!VIRT || pending < 0) return;
        const int g = pending;
        pending = -1;
        if ((tid | 63) < kBlk - mine.y) return;  // whole waves take part: finish_rows talks across lanes
        using lds_f4 = __attribute__((address_space(3))) f32x4;
        const int row0 = g * kRows;
        const int nlive = min(kRows, A - row0);
        float sum[kRows] = {0.0f, 0.0f, 0.0f, 0.0f};
        const uint32_t from = part_base + (uint32_t)(g & 1) * (16u * kBlk) + 16u * (fin & 0xffffu);
        for (uint32_t p = 0; p < (fin >> 16); ++p) {
            const f32x4 v = *reinterpret_cast<const lds_f4*>(from + 16u * p);
            sum[0] += v.x;
            sum[1] += v.y;
            sum[2] += v.z;
            sum[3] += v.w;
        }
        const unsigned pos = finish_rows(sum, bj, Yout, N, j, jok, row0, nlive, lane);
        if (lane < nlive && ((pos >> lane) & 1u)) flags[row0 + lane] = 1;
    };
    auto step = [&](int t, auto Ptag) {
        constexpr int P = decltype(Ptag)::value;
        const int gi = MULTI ? t / nstage : t;
        const int s = MULTI ? t - gi * nstage : 0;
        finish_pending();
        compute(Ptag, s, std::integral_constant<int, 0>{});
        if (t + 1 < T) store_tile(P ^ 1, t + 1);
        if (t + 2 < T) {  // the row numbers come out of a register (ListWindow): asked for only now, behind the wait for tile t+1
            fetch_rows(t + 2);
            load_tile(t + 2);
        }
        compute(Ptag, s, std::integral_constant<int, 16>{});
        if (s == nstage - 1) epilogue(g0 + gi);
        __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;

    fetch_rows(0);
    load_tile(0);
    store_tile(0, 0);
    if (T > 1) {
        fetch_rows(1);
        load_tile(1);
    }
    __syncthreads();
    int t = 0;
    for (; t + 1 < T; t += 2) {
        step(t, P0{});
        step(t + 1, P1{});
    }
    if (t < T) step(t, P0{});
    finish_pending();  // the last group (behind the last step's barrier)
}

// ---------------------------------------------------------------------------
// a1 for layers whose connections all carry the same weight (the challenge networks:
// 1/16 everywhere) and whose windows allow it: two output neurons per lane.
//
// With the weight in a scalar register a neuron needs 32 registers instead of 64, so
// a lane takes neurons j and j + 1024 of a 2048-neuron unit (output blocks 2u and
// 2u+1, set up with one common window and one common tile layout).  A staged tile
// then serves 2048 outputs: half the tile loads, LDS tile writes and L2 -> CU bytes
// per output.  Same pipeline as fused_layer_kernel<false>; nunit = number of units.
//
// RELABEL: the layer was set up under new names for neurons and columns (PairRelabel): the unit's 2048
// neurons are segments of neighbours at a stride (unit_neuron) and its tile holds the groups of four columns
// the unit reads, wherever they lie in the row.  Only what touches global memory knows: the staging lanes'
// load offsets come from the list of those groups, and bias and output addresses use the neurons' real numbers.
// ---------------------------------------------------------------------------
struct PairRelabel {
    const int32_t* col;  // [N / 4] first real column of the group of four columns that carries the new name 4g .. 4g+3
    int seg_log2;        // a unit's neurons: segments of 1 << seg_log2 neighbours, one every seg_stride neurons
    int seg_stride;
};
template <bool RELABEL = false>
__global__ __launch_bounds__(kBlk) void fused_pair_kernel(
    const float* __restrict__ Yin, float* __restrict__ Yout, uint8_t* __restrict__ flags,
    RowLists rl, LayerWeights w,
    const float* __restrict__ bias, int N, int nunit, int G, int Q, float wuni, PairRelabel rn = PairRelabel{}) {
    extern __shared__ float4 lds4[];
    const int tid = threadIdx.x;
    WorkItem wi;
    __shared__ int rl_red[17], rl_scan[17];
    if (!derive_work(rl, nunit, G, Q, wi, kRows, rl_red, rl_scan)) return;
    const int* cat = rl.cat;      // my slice of it was written just now
    const int u = wi.cb, A = wi.A, g0 = wi.g0, g1 = wi.g1;
    const int b = 2 * u;  // first of the unit's two output blocks

    // my two neurons (N is a multiple of 2048 here: both exist); four neighbouring lanes hold four neighbouring neurons
    const int jA = RELABEL ? unit_neuron(u, tid, rn.seg_log2, rn.seg_stride) : b * kBlk + tid;
    const int jB = RELABEL ? unit_neuron(u, kBlk + tid, rn.seg_log2, rn.seg_stride) : jA + kBlk;
    const int2 win = w.win[b];
    const int c_lo = win.x;
    const int ncols = win.y;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds4;

    uint32_t offA[kNnz], offB[kNnz];
    {
        const uint16_t* prel = w.rel + (size_t)b * kNnz * kBlk + tid;
#pragma unroll
        for (int k = 0; k < kNnz; ++k) {
            offA[k] = lds_base + tile_offset(prel[k * kBlk]);
            offB[k] = lds_base + tile_offset(prel[(kNnz + k) * kBlk]);
        }
    }
    const float bjA = bias[jA], bjB = bias[jB];

    const int T = g1 - g0;
    f32x4 st[kRows];
    const int wave_col = (tid & ~63) * 4;
    const bool staging = wave_col < ncols;  // waves whose columns lie past the window stage nothing
    const uint32_t st_addr = lds_base + tile_offset(store_group(4 * tid) << 4);
    const uint32_t qp = w.qsel[(size_t)b * kBlk + tid];
    ListWindow rows_of(cat, g0 * kRows, min(A, g1 * kRows), wi.identity);
    const int cat_last = rows_of.last();  // used by the last, ragged group only: then the list's last entry
    // byte offset of my four columns in a row; lanes past the window re-read its last columns
    const uint32_t ld_off = 4u * (uint32_t)(RELABEL ? rn.col[win_col(c_lo, min(4 * tid, ncols - 4), N) >> 2]
                                                    : win_col(c_lo, min(4 * tid, ncols - 4), N));  // windows are cyclic
    const char* ld_row[kRows] = {nullptr, nullptr, nullptr, nullptr};  // bases of the 4 rows of the tile to load (scalar)

    auto fetch_rows = [&](int t) {
        const int4 c4 = rows_of.get4((g0 + t) * kRows);
        const int row0 = (g0 + t) * kRows;
        ld_row[0] = reinterpret_cast<const char*>(Yin + (size_t)c4.x * N);
        ld_row[1] = reinterpret_cast<const char*>(Yin + (size_t)(row0 + 1 < A ? c4.y : cat_last) * N);
        ld_row[2] = reinterpret_cast<const char*>(Yin + (size_t)(row0 + 2 < A ? c4.z : cat_last) * N);
        ld_row[3] = reinterpret_cast<const char*>(Yin + (size_t)(row0 + 3 < A ? c4.w : cat_last) * N);
    };
    // One 16-byte load per lane and row: scalar row base + 32-bit lane offset, written as an instruction so that
    // no vector register is spent on addresses and the compiler places no wait of its own; the wait is written
    // out before the values are first touched (wait_tile).  The build checks that this kernel never spills:
    // the compiler does not know that the loaded values arrive late.
    auto load_row = [&](int r) {
        if (staging) asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(st[r]) : "v"(ld_off), "s"(ld_row[r]) : "memory");
    };
    auto wait_tile = [&]() {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        asm volatile("" : "+v"(st[0]), "+v"(st[1]), "+v"(st[2]), "+v"(st[3]));
    };
    auto store_tile = [&](int P) {
        // The four store addresses are worked out per tile, not ahead of the loop: two registers (st_addr, qp)
        // stay live instead of four, for eight cheap instructions per tile.
        uint32_t q = qp, a = st_addr;
        asm volatile("" : "+v"(q), "+v"(a));
        if (staging) stage_store(st, a + P * kBufSkew, q);
    };

    float accA[kRows] = {0.f, 0.f, 0.f, 0.f}, accB[kRows] = {0.f, 0.f, 0.f, 0.f};
    {
        const int pw = __builtin_amdgcn_readfirstlane(3 - ((threadIdx.x >> 8) & 3));
        if (pw == 1) __builtin_amdgcn_s_setprio(1);
        else if (pw == 2) __builtin_amdgcn_s_setprio(2);
        else if (pw == 3) __builtin_amdgcn_s_setprio(3);
    }
    auto compute = [&](auto Ptag, float (&acc)[kRows], const uint32_t (&off)[kNnz], auto Ktag) {
        constexpr int P = decltype(Ptag)::value;
        constexpr int k0 = decltype(Ktag)::value;
        uint32_t o[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) o[i] = off[k0 + i];
        fma_block16s<P>(acc, o, wuni);
    };

    const int lane = tid & 63;
    auto finish = [&](float (&acc)[kRows], float bj, int j, int row0, int nlive) -> unsigned {
        return finish_rows(acc, bj, Yout, N, j, true, row0, nlive, lane);
    };

    // One step: neuron A's 32 connections; tile t+1 into the other buffer; neuron B's 32 connections with the
    // loads of tile t+2 in two bursts before its two halves (a wave that issues loads is stuck until the memory
    // pipeline has taken them, and four loads per lane back to back leave the last wave some 3000 clocks behind
    // the first); both epilogues.
    using K0 = std::integral_constant<int, 0>;
    using K16 = std::integral_constant<int, 16>;
    auto step = [&](int t, auto Ptag) {
        constexpr int P = decltype(Ptag)::value;
        const bool more = t + 2 < T;
        compute(Ptag, accA, offA, K0{});
        compute(Ptag, accA, offA, K16{});
        if (t + 1 < T) {
            wait_tile();
            store_tile(P ^ 1);
        }
        if (more) {
            fetch_rows(t + 2);
            load_row(0);
            load_row(1);
        }
        compute(Ptag, accB, offB, K0{});
        if (more) {
            load_row(2);
            load_row(3);
        }
        compute(Ptag, accB, offB, K16{});
        const int row0 = (g0 + t) * kRows;
        const int nlive = min(kRows, A - row0);
        const unsigned pos = finish(accA, bjA, jA, row0, nlive) | finish(accB, bjB, jB, row0, nlive);
        if (lane < nlive && ((pos >> lane) & 1u)) flags[row0 + lane] = 1;
        __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;
    fetch_rows(0);
#pragma unroll
    for (int r = 0; r < kRows; ++r) load_row(r);
    wait_tile();
    store_tile(0);
    if (T > 1) {
        fetch_rows(1);
#pragma unroll
        for (int r = 0; r < kRows; ++r) load_row(r);
    }
    __syncthreads();
    int t = 0;
    for (; t + 1 < T; t += 2) {
        step(t, P0{});
        step(t + 1, P1{});
    }
    if (t < T) step(t, P0{});
}

// ---------------------------------------------------------------------------
// a1 for wide layers.  Same tile pipeline as fused_layer_kernel, other loop order:
// a workgroup takes kChunk row groups (32 rows), keeps their 32 accumulators per
// lane in registers and walks the stages; in each stage it loads that stage's S
// (column, weight) pairs into registers once and applies them to the chunk's 8
// tiles.  A stage thus costs S steps instead of 32, and the stage's weights are
// read once per 32 rows.
// ---------------------------------------------------------------------------
template <int S>
__global__ __launch_bounds__(kBlk) void fused_wide_kernel(
    const float* __restrict__ Yin, float* __restrict__ Yout, uint8_t* __restrict__ flags,
    RowLists rl, WideWeights w,
    const float* __restrict__ bias, int N, int nblk, int G, int Q) {
    extern __shared__ float4 lds4[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    WorkItem wi;
    __shared__ int rl_red[17], rl_scan[17];
    if (!derive_work(rl, nblk, G, Q, wi, kRows, rl_red, rl_scan)) return;
    const int* cat = rl.cat;      // my slice of it was written just now
    const int b = wi.cb, A = wi.A, g0 = wi.g0, g1 = wi.g1;

    const int j = b * kBlk + tid;
    const bool jok = j < N;
    const int2 win = w.win[b];
    const int c_lo = win.x;
    const int ncols = win.y;
    const int nstage = w.nstage;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds4;
    const float bj = jok ? bias[j] : 0.0f;

    const int nchunk = (g1 - g0 + kChunk - 1) / kChunk;
    const int per_chunk = nstage * kChunk;
    const int T = nchunk * per_chunk;  // steps: (chunk, stage, tile); tiles past g1 repeat the last group

    f32x4 st[kRows];
    const int wave_col = (tid & ~63) * 4;
    const uint32_t st_addr = lds_base + tile_offset(col_slot(4 * tid));
    ListWindow rows_of(cat, g0 * kRows, min(A, g1 * kRows), wi.identity);
    const int cat_last = rows_of.last();  // used by the last, ragged group only: then the list's last entry
    int4 c4 = make_int4(0, 0, 0, 0);

    auto group_of = [&](int t, int& s) -> int {
        const int c = t / per_chunk;
        const int rem = t - c * per_chunk;
        s = rem / kChunk;
        return min(g0 + c * kChunk + (rem - s * kChunk), g1 - 1);
    };
    auto fetch_rows = [&](int t) {
        int s;
        const int g = group_of(t, s);
        c4 = rows_of.get4(g * kRows);
    };
    auto load_tile = [&](int t) {
        int s;
        const int g = group_of(t, s);
        const int left = ncols - s * kCap;
        if (wave_col >= left) return;
        const int row0 = g * kRows;
        const size_t coff = (size_t)win_col(c_lo, s * kCap + min(4 * tid, left - 4), N);  // windows are cyclic
        stage_load(st, Yin, N, c4, row0, A, cat_last, coff);
    };
    auto store_tile = [&](int P, int t) {
        int s;
        (void)group_of(t, s);
        const int left = ncols - s * kCap;
        if (wave_col >= left) return;
        stage_store(st, st_addr + P * kBufSkew, 0u);
    };

    float acc[kChunk][kRows];
#pragma unroll
    for (int i = 0; i < kChunk; ++i)
#pragma unroll
        for (int r = 0; r < kRows; ++r) acc[i][r] = 0.0f;

    uint32_t ow[S];
    float wv[S];
    int nb = 0;  // blocks of 8 steps my wave needs in the current stage
    auto load_weights = [&](int s) {
        const uint4* p = reinterpret_cast<const uint4*>(w.pk) + ((size_t)(b * nstage + s) * (S / 2)) * kBlk + tid;
#pragma unroll
        for (int k2 = 0; k2 < S / 2; ++k2) {
            const uint4 v = p[(size_t)k2 * kBlk];
            ow[2 * k2] = lds_base + tile_offset(v.x);
            wv[2 * k2] = __builtin_bit_cast(float, v.y);
            ow[2 * k2 + 1] = lds_base + tile_offset(v.z);
            wv[2 * k2 + 1] = __builtin_bit_cast(float, v.w);
        }
        nb = w.nb8[(b * nstage + s) * 16 + wave];
    };

    const int nspill = w.spill_n[b * 16 + wave];
    auto epilogue = [&](int g, float (&a)[kRows]) {
        const int row0 = g * kRows;
        const int nlive = min(kRows, A - row0);
        if (nspill > 0) {  // connections that did not fit a stage: gathered from global memory
            const int4 cg = wi.identity ? make_int4(row0, row0 + 1, row0 + 2, row0 + 3)
                                        : uniform4(*reinterpret_cast<const int4*>(cat + (size_t)g * kRows));
            const float* p0 = Yin + (size_t)cg.x * N;
            const float* p1 = Yin + (size_t)(nlive > 1 ? cg.y : cat_last) * N;
            const float* p2 = Yin + (size_t)(nlive > 2 ? cg.z : cat_last) * N;
            const float* p3 = Yin + (size_t)(nlive > 3 ? cg.w : cat_last) * N;
            for (int e = 0; e < nspill; ++e) {
                const size_t se = ((size_t)b * kSpill + e) * kBlk + tid;
                const int col = win_col(c_lo, w.spill_col[se], N);  // windows are cyclic
                const float v = w.spill_val[se];
                a[0] = __builtin_fmaf(p0[col], v, a[0]);
                a[1] = __builtin_fmaf(p1[col], v, a[1]);
                a[2] = __builtin_fmaf(p2[col], v, a[2]);
                a[3] = __builtin_fmaf(p3[col], v, a[3]);
            }
        }
        const float y0 = fminf(fmaxf(a[0] + bj, 0.0f), kClip);
        const float y1 = fminf(fmaxf(a[1] + bj, 0.0f), kClip);
        const float y2 = fminf(fmaxf(a[2] + bj, 0.0f), kClip);
        const float y3 = fminf(fmaxf(a[3] + bj, 0.0f), kClip);
        a[0] = a[1] = a[2] = a[3] = 0.0f;
        const unsigned pos = (__builtin_amdgcn_ballot_w64(y0 > 0.0f) != 0ull ? 1u : 0u) |
                             (__builtin_amdgcn_ballot_w64(y1 > 0.0f) != 0ull ? 2u : 0u) |
                             (__builtin_amdgcn_ballot_w64(y2 > 0.0f) != 0ull ? 4u : 0u) |
                             (__builtin_amdgcn_ballot_w64(y3 > 0.0f) != 0ull ? 8u : 0u);
        if (lane < nlive && ((pos >> lane) & 1u)) flags[row0 + lane] = 1;
        if (jok) {
            float* dst = Yout + (size_t)row0 * N + j;
            dst[0] = y0;
            if (nlive > 1) dst[(size_t)N] = y1;
            if (nlive > 2) dst[2 * (size_t)N] = y2;
            if (nlive > 3) dst[3 * (size_t)N] = y3;
        }
    };

    // One step: the first 8 connections of the stage, the next tile into the other LDS
    // buffer and the loads of the tile after it, then the other 8 connections.
    auto step = [&](int t, auto Ptag, float (&a)[kRows]) {
        constexpr int P = decltype(Ptag)::value;
        if (nb > 0) {
            uint32_t o8[8];
            float v8[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                o8[k] = ow[k];
                v8[k] = wv[k];
            }
            fma_block8<P>(a, o8, v8);
        }
        if (t + 1 < T) store_tile(P ^ 1, t + 1);
        if (t + 2 < T) {  // the row numbers come out of a register (ListWindow): asked for only now, behind the wait for tile t+1
            fetch_rows(t + 2);
            load_tile(t + 2);
        }
        if (S > 8 && nb > 1) {
            uint32_t o8[8];
            float v8[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                o8[k] = ow[(S > 8 ? 8 : 0) + k];
                v8[k] = wv[(S > 8 ? 8 : 0) + k];
            }
            fma_block8<P>(a, o8, v8);
        }
        __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;

    fetch_rows(0);
    load_tile(0);
    store_tile(0, 0);
    fetch_rows(1);
    load_tile(1);
    __syncthreads();
    int t = 0;
    for (int c = 0; c < nchunk; ++c) {
        for (int s = 0; s < nstage; ++s) {
            load_weights(s);
#pragma unroll
            for (int i = 0; i < kChunk; i += 2) {
                step(t, P0{}, acc[i]);
                step(t + 1, P1{}, acc[i + 1]);
                t += 2;
            }
        }
        // all stages applied: bias, clip, store and row flags of the chunk's row groups
        const int gbase = g0 + c * kChunk;
#pragma unroll
        for (int i = 0; i < kChunk; ++i)
            if (gbase + i < g1) epilogue(gbase + i, acc[i]);
    }
}

// ---------------------------------------------------------------------------
// a1 for wide layers with one weight for the whole layer: two output neurons per lane
// (j and j + 1024 of a 2048-neuron unit), as in fused_pair_kernel.  The stage's
// connections are read in a compact form (16-bit LDS slots, no weights), a step that a
// neuron does not fill reads an all-zero LDS entry kept behind the tile pair, and a
// chunk is kChunkPair = 4 row groups so that the 32 accumulators per lane stay.  Every
// staged tile serves 2048 outputs: half the tile traffic per output of
// fused_wide_kernel.  S = 16 steps per stage only (3 to 8 stages).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlk) void fused_wide_pair_kernel(
    const float* __restrict__ Yin, float* __restrict__ Yout, uint8_t* __restrict__ flags,
    RowLists rl, WideWeights w,
    const float* __restrict__ bias, int N, int nunit, int G, int Q, float wuni) {
    constexpr int S = 16;
    extern __shared__ float4 lds4[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    WorkItem wi;
    __shared__ int rl_red[17], rl_scan[17];
    if (!derive_work(rl, nunit, G, Q, wi, kRows, rl_red, rl_scan)) return;
    const int* cat = rl.cat;      // my slice of it was written just now
    const int u = wi.cb, A = wi.A, g0 = wi.g0, g1 = wi.g1;
    const int b = 2 * u;  // first of the unit's two output blocks (same window for both)

    const int jA = b * kBlk + tid, jB = jA + kBlk;  // N is a multiple of 2048 here
    const int2 win = w.win[b];
    const int c_lo = win.x;
    const int ncols = win.y;
    const int nstage = w.nstage;
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds4;
    // 512 zero bytes behind the tile pair: slots kCap .. kCap+15, an entry per bank quad, for either buffer
    const uint32_t zero_addr = lds_base + tile_pair_bytes(kCap);
    if (tid < 2 * kBufSkew / 16) {
        using lds_f4 = __attribute__((address_space(3))) f32x4;
        *reinterpret_cast<lds_f4*>(zero_addr + tid * 16) = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const float bjA = bias[jA], bjB = bias[jB];

    const int nchunk = (g1 - g0 + kChunkPair - 1) / kChunkPair;
    const int per_chunk = nstage * kChunkPair;
    const int T = nchunk * per_chunk;  // steps: (chunk, stage, tile); tiles past g1 repeat the last group

    f32x4 st[kRows];
    const int wave_col = (tid & ~63) * 4;
    const uint32_t st_addr = lds_base + tile_offset(col_slot(4 * tid));
    ListWindow rows_of(cat, g0 * kRows, min(A, g1 * kRows), wi.identity);
    const int cat_last = rows_of.last();  // used by the last, ragged group only: then the list's last entry
    int4 c4 = make_int4(0, 0, 0, 0);

    auto group_of = [&](int t, int& s) -> int {
        const int c = t / per_chunk;
        const int rem = t - c * per_chunk;
        s = rem / kChunkPair;
        return min(g0 + c * kChunkPair + (rem - s * kChunkPair), g1 - 1);
    };
    auto fetch_rows = [&](int t) {
        int s;
        const int g = group_of(t, s);
        c4 = rows_of.get4(g * kRows);
    };
    auto load_tile = [&](int t) {
        int s;
        const int g = group_of(t, s);
        const int left = ncols - s * kCap;
        if (wave_col >= left) return;
        const int row0 = g * kRows;
        const size_t coff = (size_t)win_col(c_lo, s * kCap + min(4 * tid, left - 4), N);  // windows are cyclic
        stage_load(st, Yin, N, c4, row0, A, cat_last, coff);
    };
    auto store_tile = [&](int P, int t) {
        int s;
        (void)group_of(t, s);
        const int left = ncols - s * kCap;
        if (wave_col >= left) return;
        stage_store(st, st_addr + P * kBufSkew, 0u);
    };

    float accA[kChunkPair][kRows], accB[kChunkPair][kRows];
#pragma unroll
    for (int i = 0; i < kChunkPair; ++i)
#pragma unroll
        for (int r = 0; r < kRows; ++r) accA[i][r] = accB[i][r] = 0.0f;

    uint32_t owA[S], owB[S];
    int nbA = 0, nbB = 0;  // blocks of 8 steps my wave needs in the current stage, per neuron
    auto unpack8 = [&](const uint4 v, uint32_t* o) {
        const uint32_t x[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t lo = x[i] & 0xFFFFu, hi = x[i] >> 16;
            o[2 * i] = lds_base + tile_offset(lo);  // padding codes are slots of the zero entries
            o[2 * i + 1] = lds_base + tile_offset(hi);
        }
    };
    auto load_weights = [&](int s) {
        const uint4* pA = w.ps + ((size_t)(b * nstage + s) * (S / 8)) * kBlk + tid;
        const uint4* pB = w.ps + ((size_t)((b + 1) * nstage + s) * (S / 8)) * kBlk + tid;
        unpack8(pA[0], owA);
        unpack8(pA[kBlk], owA + 8);
        unpack8(pB[0], owB);
        unpack8(pB[kBlk], owB + 8);
        nbA = w.nb8[(b * nstage + s) * 16 + wave];
        nbB = w.nb8[((b + 1) * nstage + s) * 16 + wave];
    };

    const int nspillA = w.spill_n[b * 16 + wave], nspillB = w.spill_n[(b + 1) * 16 + wave];
    // spilled connections (gathered from global memory), bias, clip, store of one neuron's 4 rows
    auto finish = [&](float (&a)[kRows], float bj, int j, int blk, int nspill, int g, int nlive) -> unsigned {
        const int row0 = g * kRows;
        if (nspill > 0) {
            const int4 cg = wi.identity ? make_int4(row0, row0 + 1, row0 + 2, row0 + 3)
                                        : uniform4(*reinterpret_cast<const int4*>(cat + (size_t)g * kRows));
            const float* p0 = Yin + (size_t)cg.x * N;
            const float* p1 = Yin + (size_t)(nlive > 1 ? cg.y : cat_last) * N;
            const float* p2 = Yin + (size_t)(nlive > 2 ? cg.z : cat_last) * N;
            const float* p3 = Yin + (size_t)(nlive > 3 ? cg.w : cat_last) * N;
            for (int e = 0; e < nspill; ++e) {
                const size_t se = ((size_t)blk * kSpill + e) * kBlk + tid;
                const int col = win_col(c_lo, w.spill_col[se], N);  // windows are cyclic
                const float v = w.spill_val[se];
                a[0] = __builtin_fmaf(p0[col], v, a[0]);
                a[1] = __builtin_fmaf(p1[col], v, a[1]);
                a[2] = __builtin_fmaf(p2[col], v, a[2]);
                a[3] = __builtin_fmaf(p3[col], v, a[3]);
            }
        }
        const float y0 = fminf(fmaxf(a[0] + bj, 0.0f), kClip);
        const float y1 = fminf(fmaxf(a[1] + bj, 0.0f), kClip);
        const float y2 = fminf(fmaxf(a[2] + bj, 0.0f), kClip);
        const float y3 = fminf(fmaxf(a[3] + bj, 0.0f), kClip);
        a[0] = a[1] = a[2] = a[3] = 0.0f;
        const unsigned pos = (__builtin_amdgcn_ballot_w64(y0 > 0.0f) != 0ull ? 1u : 0u) |
                             (__builtin_amdgcn_ballot_w64(y1 > 0.0f) != 0ull ? 2u : 0u) |
                             (__builtin_amdgcn_ballot_w64(y2 > 0.0f) != 0ull ? 4u : 0u) |
                             (__builtin_amdgcn_ballot_w64(y3 > 0.0f) != 0ull ? 8u : 0u);
        float* dst = Yout + (size_t)row0 * N + j;
        dst[0] = y0;
        if (nlive > 1) dst[(size_t)N] = y1;
        if (nlive > 2) dst[2 * (size_t)N] = y2;
        if (nlive > 3) dst[3 * (size_t)N] = y3;
        return pos;
    };

    auto block = [&](auto Ptag, float (&a)[kRows], const uint32_t* o) {
        constexpr int P = decltype(Ptag)::value;
        uint32_t o8[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) o8[k] = o[k];
        fma_block8s<P>(a, o8, wuni);
    };
    // One step: neuron A's first 8 steps of the stage, the next tile into the other LDS
    // buffer and the loads of the tile after it, then A's other 8 and B's 16.
    auto step = [&](int t, auto Ptag, float (&aA)[kRows], float (&aB)[kRows]) {
        constexpr int P = decltype(Ptag)::value;
        if (nbA > 0) block(Ptag, aA, owA);
        if (t + 1 < T) store_tile(P ^ 1, t + 1);
        if (t + 2 < T) {  // the row numbers come out of a register (ListWindow): asked for only now, behind the wait for tile t+1
            fetch_rows(t + 2);
            load_tile(t + 2);
        }
        if (nbA > 1) block(Ptag, aA, owA + 8);
        if (nbB > 0) block(Ptag, aB, owB);
        if (nbB > 1) block(Ptag, aB, owB + 8);
        __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;

    fetch_rows(0);
    load_tile(0);
    store_tile(0, 0);
    fetch_rows(1);
    load_tile(1);
    __syncthreads();
    int t = 0;
    for (int c = 0; c < nchunk; ++c) {
        for (int s = 0; s < nstage; ++s) {
            load_weights(s);
#pragma unroll
            for (int i = 0; i < kChunkPair; i += 2) {
                step(t, P0{}, accA[i], accB[i]);
                step(t + 1, P1{}, accA[i + 1], accB[i + 1]);
                t += 2;
            }
        }
        const int gbase = g0 + c * kChunkPair;
#pragma unroll
        for (int i = 0; i < kChunkPair; ++i)
            if (gbase + i < g1) {
                const int g = gbase + i;
                const int nlive = min(kRows, A - g * kRows);
                const unsigned pos = finish(accA[i], bjA, jA, b, nspillA, g, nlive) |
                                     finish(accB[i], bjB, jB, b + 1, nspillB, g, nlive);
                if (lane < nlive && ((pos >> lane) & 1u)) flags[g * kRows + lane] = 1;
            }
    }
}

// ---------------------------------------------------------------------------
// a1 for wide layers of 2 to 4 stages with one weight for the whole layer: two output
// neurons per lane with the slot lists of ALL stages resident in registers (two 16-bit
// LDS addresses per register: 4 stages x 16 steps, or 2 stages x 32 steps, x 2 neurons =
// 64 registers), so that
// nothing but tiles is read inside the loop and a stage never waits for its step list.
// A step is (row group, stage); every row group takes 4 steps (the last one idle when
// there are 3 stages, which keeps the tile buffers alternating).  Unused steps read the
// all-zero entry behind the tile pair.  The connections beyond the 16 steps of a stage
// (up to kSpill per neuron) sit in a small LDS table and are read from the tile in their
// stage's step like the others.
// ---------------------------------------------------------------------------
template <int NS, int S>
__global__ __launch_bounds__(kBlk) void fused_wide_pair4_kernel(
    const float* __restrict__ Yin, float* __restrict__ Yout, uint8_t* __restrict__ flags,
    RowLists rl, WideWeights w,
    const float* __restrict__ bias, int N, int nunit, int G, int Q, float wuni) {
    static_assert(NS * S == 64 && (NS == 2 || NS == 4), "64 steps per neuron");
    constexpr int LNS = NS == 4 ? 2 : 1;  // log2(NS)
    extern __shared__ float4 lds4[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    WorkItem wi;
    __shared__ int rl_red[17], rl_scan[17];
    if (!derive_work(rl, nunit, G, Q, wi, kRows, rl_red, rl_scan)) return;
    const int* cat = rl.cat;      // my slice of it was written just now
    const int u = wi.cb, A = wi.A, g0 = wi.g0, g1 = wi.g1;
    const int b = 2 * u;

    const int jA = b * kBlk + tid;  // neuron B is jA + kBlk; N is a multiple of 2048 here
    const int2 win = w.win[b];
    const int c_lo = win.x;
    const int ncols = win.y;
    const int nstage = w.nstage;  // NS = 4: 3 or 4; NS = 2: 2
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds4;
    // 512 zero bytes behind the tile pair: slots kCap .. kCap+15, an entry per bank quad, for either buffer
    const uint32_t zero_addr = lds_base + tile_pair_bytes(kCap);
    if (tid < 2 * kBufSkew / 16) {
        using lds_f4 = __attribute__((address_space(3))) f32x4;
        *reinterpret_cast<lds_f4*>(zero_addr + tid * 16) = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const float bjA = bias[jA], bjB = bias[jA + kBlk];
    uint32_t sh4 = 4;
    asm volatile("" : "+s"(sh4));  // the shift count of fma_block8ps, kept in a scalar register

    // step lists of both neurons, all stages: word i of stage s = steps 2i, 2i+1 as (LDS byte address >> 4)
    uint32_t pA[NS * S / 2], pB[NS * S / 2];
    int nbA[NS], nbB[NS];  // blocks of 8 steps my wave needs per stage and neuron
    {
        const uint32_t zero16 = zero_addr >> 4, base16 = lds_base >> 4;
        auto conv = [&](uint32_t two) -> uint32_t {
            const uint32_t lo = two & 0xFFFFu, hi = two >> 16;
            const uint32_t a = base16 + (tile_offset(lo) >> 4);  // padding codes are slots of the zero entries
            const uint32_t c = base16 + (tile_offset(hi) >> 4);
            return a | (c << 16);
        };
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            if (s < nstage) {
                const uint4* qA = w.ps + ((size_t)(b * nstage + s) * (S / 8)) * kBlk + tid;
                const uint4* qB = w.ps + ((size_t)((b + 1) * nstage + s) * (S / 8)) * kBlk + tid;
#pragma unroll
                for (int o = 0; o < S / 8; ++o) {
                    const uint4 va = qA[o * kBlk], vb = qB[o * kBlk];
                    pA[s * (S / 2) + o * 4 + 0] = conv(va.x);
                    pA[s * (S / 2) + o * 4 + 1] = conv(va.y);
                    pA[s * (S / 2) + o * 4 + 2] = conv(va.z);
                    pA[s * (S / 2) + o * 4 + 3] = conv(va.w);
                    pB[s * (S / 2) + o * 4 + 0] = conv(vb.x);
                    pB[s * (S / 2) + o * 4 + 1] = conv(vb.y);
                    pB[s * (S / 2) + o * 4 + 2] = conv(vb.z);
                    pB[s * (S / 2) + o * 4 + 3] = conv(vb.w);
                }
                nbA[s] = __builtin_amdgcn_readfirstlane((int)w.nb8[(b * nstage + s) * 16 + wave]);
                nbB[s] = __builtin_amdgcn_readfirstlane((int)w.nb8[((b + 1) * nstage + s) * 16 + wave]);
            } else {
#pragma unroll
                for (int i = 0; i < S / 2; ++i) pA[s * (S / 2) + i] = pB[s * (S / 2) + i] = zero16 | (zero16 << 16);
                nbA[s] = nbB[s] = 0;
            }
        }
    }

    // Spilled connections: entry e of neuron A (B) of lane t at spill_tab + ((2e (+1)) * kBlk + t) * 2,
    // stage << 14 | (LDS byte address >> 4), 0xFFFF = none.
    const uint32_t spill_tab = zero_addr + 2 * kBufSkew;
    const int nspillA = w.spill_n[b * 16 + wave], nspillB = w.spill_n[(b + 1) * 16 + wave];
    bool anyA[NS] = {}, anyB[NS] = {};
    {
        using lds_u16 = __attribute__((address_space(3))) uint16_t;
#pragma unroll
        for (int e = 0; e < kSpill; ++e) {
            const uint32_t va = w.sp16[((size_t)b * kSpill + e) * kBlk + tid];
            const uint32_t vb = w.sp16[((size_t)(b + 1) * kSpill + e) * kBlk + tid];
            *reinterpret_cast<lds_u16*>(spill_tab + ((2 * e) * kBlk + tid) * 2) = (uint16_t)va;
            *reinterpret_cast<lds_u16*>(spill_tab + ((2 * e + 1) * kBlk + tid) * 2) = (uint16_t)vb;
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                anyA[s] = anyA[s] || __builtin_amdgcn_ballot_w64(va != 0xFFFFu && (va >> 14) == (uint32_t)s) != 0ull;
                anyB[s] = anyB[s] || __builtin_amdgcn_ballot_w64(vb != 0xFFFFu && (vb >> 14) == (uint32_t)s) != 0ull;
            }
        }
    }
    auto spilled = [&](auto Ptag, float (&acc)[kRows], int which, int nspill, int s) {
        constexpr int P = decltype(Ptag)::value;
        using lds_f4 = __attribute__((address_space(3))) f32x4;
        using lds_u16 = __attribute__((address_space(3))) uint16_t;
        for (int e = 0; e < nspill; ++e) {
            const uint32_t v = *reinterpret_cast<const lds_u16*>(spill_tab + ((2 * e + which) * kBlk + tid) * 2);
            const uint32_t addr = (v != 0xFFFFu && (v >> 14) == (uint32_t)s) ? lds_base + ((v & 0x3FFFu) << 4) : zero_addr;
            const f32x4 y = *reinterpret_cast<const lds_f4*>(addr + P * kBufSkew);
            acc[0] = __builtin_fmaf(y.x, wuni, acc[0]);
            acc[1] = __builtin_fmaf(y.y, wuni, acc[1]);
            acc[2] = __builtin_fmaf(y.z, wuni, acc[2]);
            acc[3] = __builtin_fmaf(y.w, wuni, acc[3]);
        }
    };

    const int T = (g1 - g0) * NS;  // steps; step t = (row group t / NS, stage t % NS)
    f32x4 st[kRows];
    const int wave_col = (tid & ~63) * 4;
    const uint32_t st_addr = lds_base + tile_offset(col_slot(4 * tid));
    ListWindow rows_of(cat, g0 * kRows, min(A, g1 * kRows), wi.identity);
    const int cat_last = rows_of.last();  // used by the last, ragged group only: then the list's last entry
    int4 c4 = make_int4(0, 0, 0, 0);

    auto fetch_rows = [&](int t) { c4 = rows_of.get4((g0 + (t >> LNS)) * kRows); };
    // column (in floats) of my four staged columns: the same in every full stage, clamped in a narrower last one
    const uint32_t col_full = (uint32_t)(c_lo + 4 * tid);
    const uint32_t col_last = (uint32_t)(c_lo + (nstage - 1) * kCap + min(4 * tid, ncols - (nstage - 1) * kCap - 4));
    auto load_tile = [&](int t) {
        const int s = t & (NS - 1);
        const int left = ncols - s * kCap;  // <= 0 for the idle fourth step of a 3-stage layer
        if (wave_col >= left) return;
        const int row0 = (g0 + (t >> LNS)) * kRows;
        uint32_t col = s == nstage - 1 ? col_last : col_full + (uint32_t)(s * kCap);
        if (col >= (uint32_t)N) col -= (uint32_t)N;  // windows are cyclic
        const float* r0 = Yin + (size_t)c4.x * N;  // row bases are the same for the whole workgroup
        const float* r1 = Yin + (size_t)(row0 + 1 < A ? c4.y : cat_last) * N;
        const float* r2 = Yin + (size_t)(row0 + 2 < A ? c4.z : cat_last) * N;
        const float* r3 = Yin + (size_t)(row0 + 3 < A ? c4.w : cat_last) * N;
        st[0] = *reinterpret_cast<const f32x4*>(r0 + col);
        st[1] = *reinterpret_cast<const f32x4*>(r1 + col);
        st[2] = *reinterpret_cast<const f32x4*>(r2 + col);
        st[3] = *reinterpret_cast<const f32x4*>(r3 + col);
    };
    auto store_tile = [&](int P, int t) {
        const int left = ncols - (t & (NS - 1)) * kCap;
        if (wave_col >= left) return;
        stage_store(st, st_addr + P * kBufSkew, 0u);
    };

    float accA[kRows] = {0.f, 0.f, 0.f, 0.f}, accB[kRows] = {0.f, 0.f, 0.f, 0.f};
    auto finish = [&](float (&a)[kRows], float bj, int j, int g, int nlive) -> unsigned {
        return finish_rows(a, bj, Yout, N, j, true, g * kRows, nlive, lane);
    };

    // One step with compile-time tile buffer P and stage s.
    auto step = [&](int t, auto Ptag, auto Stag) {
        constexpr int P = decltype(Ptag)::value;
        constexpr int s = decltype(Stag)::value;
        constexpr int o = s * (S / 2);  // first word of this stage's steps
        if (nbA[s] > 0) fma_block8ps<P>(accA, pA[o + 0], pA[o + 1], pA[o + 2], pA[o + 3], wuni, sh4);
        if (t + 1 < T) store_tile(P ^ 1, t + 1);
        if (t + 2 < T) {  // the row numbers come out of a register (ListWindow): asked for only now, behind the wait for tile t+1
            fetch_rows(t + 2);
            load_tile(t + 2);
        }
#pragma unroll
        for (int blk = 1; blk < S / 8; ++blk)
            if (nbA[s] > blk) fma_block8ps<P>(accA, pA[o + 4 * blk], pA[o + 4 * blk + 1], pA[o + 4 * blk + 2], pA[o + 4 * blk + 3], wuni, sh4);
#pragma unroll
        for (int blk = 0; blk < S / 8; ++blk)
            if (nbB[s] > blk) fma_block8ps<P>(accB, pB[o + 4 * blk], pB[o + 4 * blk + 1], pB[o + 4 * blk + 2], pB[o + 4 * blk + 3], wuni, sh4);
        if (anyA[s]) spilled(Ptag, accA, 0, nspillA, s);
        if (anyB[s]) spilled(Ptag, accB, 1, nspillB, s);
        if (s >= NS - 2 && s == nstage - 1) {  // s is a compile-time constant: no epilogue code in the steps that cannot be last
            const int g = g0 + (t >> LNS);
            const int nlive = min(kRows, A - g * kRows);
            const unsigned pos = finish(accA, bjA, jA, g, nlive) | finish(accB, bjB, jA + kBlk, g, nlive);
            if (lane < nlive && ((pos >> lane) & 1u)) flags[g * kRows + lane] = 1;
        }
        __syncthreads();
    };
    using P0 = std::integral_constant<int, 0>;
    using P1 = std::integral_constant<int, 1>;

    fetch_rows(0);
    load_tile(0);
    store_tile(0, 0);
    fetch_rows(1);
    load_tile(1);
    __syncthreads();
    for (int t = 0; t < T; t += NS) {
        step(t, P0{}, std::integral_constant<int, 0>{});
        step(t + 1, P1{}, std::integral_constant<int, 1>{});
        if constexpr (NS == 4) {
            step(t + 2, P0{}, std::integral_constant<int, 2>{});
            step(t + 3, P1{}, std::integral_constant<int, 3>{});
        }
    }
}

}  // namespace spdnn
#include "spdnn_row2.h"
#include "spdnn_chain.h"
namespace spdnn {

// Compact form of a wide layer's steps for the two-neurons-per-lane wide kernels: the 16-bit
// LDS slot of every step, 0xFFFF where the step carries no connection (weight 0 in pk).  One
// thread per 16-byte output (eight steps of one lane); S = steps per stage (16 or 32).
__global__ void wide_slots_kernel(const uint2* __restrict__ pk, uint4* __restrict__ ps, size_t n_out, int S) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // = ((block*nstage + stage)*(S/8) + octet)*kBlk + lane
    if (i >= n_out) return;
    const size_t lane = i % kBlk, bo = i / kBlk;
    const size_t bs = bo / (S / 8), octet = bo % (S / 8);  // bs = block*nstage + stage
    uint32_t h[8];
    for (int k = 0; k < 8; ++k) {
        // step 8*octet + k of this lane: pk index ((bs*(S/2) + step/2)*kBlk + lane)*2 + step%2
        const size_t step = 8 * octet + k;
        const uint2 e = pk[(((bs * (S / 2) + (step >> 1)) * kBlk + lane) << 1) | (step & 1)];
        h[k] = e.y != 0u ? (e.x & 0xFFFFu) : kPadSlot | (e.x & 15u);  // weight 0: zeros from the same quad
    }
    ps[i] = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
}

// Spilled connections in the form fused_wide_pair4_kernel keeps in LDS: stage << 14 | (tile byte
// offset of the column's entry >> 4), 0xFFFF where the list has no entry.  One thread per entry.
constexpr int kPadLds = 2 * kBufSkew;  // the zero entries behind the tile pair
constexpr int kPair4LdsExtra = kPadLds + 2 * kSpill * kBlk * 2;  // zero entries + spill table behind the tile pair
__global__ void wide_spill16_kernel(const uint16_t* __restrict__ spill_col, const float* __restrict__ spill_val,
                                    uint16_t* __restrict__ sp16, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;  // (block * kSpill + e) * kBlk + lane
    if (i >= n) return;
    uint32_t out = 0xFFFFu;
    if (spill_val[i] != 0.0f) {  // weight 0 = no connection
        const uint32_t rel = spill_col[i];  // column - c_lo: stage << 12 | column inside the stage
        out = ((rel >> kCapLog2) << 14) | (tile_offset(col_slot(rel & (kCap - 1))) >> 4);
    }
    sp16[i] = (uint16_t)out;
}

// ---------------------------------------------------------------------------
// a2: active-row compaction (the host loop of Listing 1 between two layers,
// moved onto the GPU).  Stable filter of the A rows whose flag is set:
// cat_out[p] = slot in the buffer just written, gid_out[p] = original row id,
// *count_out = new A.  The new count is also stored to pinned host memory so the
// host can size later launches without a stream sync.
//
// Flags are bytes (0 or 1).  kCompactWGs workgroups, no communication between them:
// workgroup w owns the rows [w*S, (w+1)*S) (S a multiple of 1024) and counts for
// itself the flags set before its slice -- at most A bytes, read 16 at a time, which is
// less than what its own slice costs -- so no workgroup ever waits for another.  Its
// own slice goes in chunks of kCompactRounds rounds of 1024 rows, three phases each so
// that no phase is a chain of dependent round trips: (1) every thread reads its flag
// and its row number of every round, remembers the flags as bits, and a wave64 ballot
// gives each wave's count per round; (2) the rounds x 16 counts are scanned once by
// the whole workgroup; (3) every thread re-derives its rank from a ballot of its
// remembered bit and writes its rows out (no loads left in this phase).
//
// Flags and count are double-buffered over the layers: this launch reads flags_in and
// count_in, which the other workgroups may still be reading, writes count_out, and
// clears the same rows of flags_clear, the buffer the next layer's kernel raises its
// flags in.  (A never grows, so rows past A in either buffer are never read again.)
// ---------------------------------------------------------------------------
constexpr int kCompactWGs = 16;
constexpr int kCompactRounds = 4;
static_assert(kCompactRounds * 16 == 64, "one wave scans the (round, wave) counts");

__global__ __launch_bounds__(1024) void compact_kernel(const uint8_t* __restrict__ flags_in,
                                                       uint8_t* __restrict__ flags_clear,
                                                       const int* __restrict__ count_in, int* __restrict__ count_out,
                                                       const int* __restrict__ gid_in, int* __restrict__ gid_out,
                                                       int* __restrict__ cat_out, int* host_count) {
    __shared__ int tot[kCompactRounds * 16];  // [round][wave]: kept rows, then exclusive offsets
    __shared__ int wave_tot[16];
    __shared__ int red[17];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int A = *count_in;
    const int S = ((A + (int)gridDim.x - 1) / (int)gridDim.x + 1023) & ~1023;
    const int lo = min(A, (int)blockIdx.x * S);
    const int hi = min(A, lo + S);
    if (blockIdx.x == 0) {  // the first workgroup also reports the new count
        const int total = count_flags(flags_in, A, red);
        if (tid == 0) {
            *count_out = total;
            __hip_atomic_store(host_count, total, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
    if (lo >= hi) return;
    int base = count_flags(flags_in, lo, red);  // rows kept before my slice (lo is a multiple of 1024)
    for (int chunk0 = lo; chunk0 < hi; chunk0 += kCompactRounds * 1024) {
        const int nr = min(kCompactRounds, (hi - chunk0 + 1023) >> 10);
        unsigned mine = 0u;
        int f[kCompactRounds], g[kCompactRounds];  // my flag and original row number of round r
#pragma unroll
        for (int r = 0; r < kCompactRounds; ++r) {
            const int i = chunk0 + (r << 10) + tid;
            const bool ok = r < nr && i < hi;
            f[r] = ok ? flags_in[i] : 0;
            g[r] = ok ? gid_in[i] : 0;
        }
#pragma unroll
        for (int r = 0; r < kCompactRounds; ++r) {
            const int i = chunk0 + (r << 10) + tid;
            if (r < nr && i < hi) flags_clear[i] = 0;
            const unsigned long long m = __ballot(f[r] != 0);
            if (f[r] != 0) mine |= 1u << r;
            if (lane == 0) tot[r * 16 + wave] = __popcll(m);
        }
        __syncthreads();
        // exclusive scan over the (round, wave) counts: entry tid = round tid/16, wave tid%16 (one wave's worth)
        if (wave == 0) {
            const int v = tot[lane];
            int incl = v;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int up = __shfl_up(incl, d, 64);
                if (lane >= d) incl += up;
            }
            tot[lane] = incl - v;
            if (lane == 63) wave_tot[0] = incl;
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < kCompactRounds; ++r) {
            const bool keep = (mine >> r) & 1u;
            const unsigned long long m = __ballot(keep);
            if (keep) {
                const int p = base + tot[r * 16 + wave] + __popcll(m & ((1ull << lane) - 1ull));
                cat_out[p] = chunk0 + (r << 10) + tid;
                gid_out[p] = g[r];
            }
        }
        base += wave_tot[0];
        __syncthreads();
    }
}

// Start of an inference, written as the state a "layer -1" would have left: all rows of the batch
// flagged alive, A = batch, the first layer's own flags cleared.  Row i of the input carries the
// original row number row_offset + i (inputs handed over in serial batches, Section III-B-2, are
// numbered through).
__global__ void init_lists_kernel(int* __restrict__ gid_prev, uint8_t* __restrict__ flags_prev,
                                  uint8_t* __restrict__ flags_first, int* __restrict__ count_prev, int batch,
                                  int row_offset, int* __restrict__ counters = nullptr, int ncounters = 0) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < batch) {
        gid_prev[i] = row_offset + i;
        flags_prev[i] = 1;
        flags_first[i] = 0;
    }
    if (i == 0) *count_prev = batch;
    // counters that the inference adds to (rows per layer of a one-launch run), cleared here
    for (int k = i; k < ncounters; k += gridDim.x * blockDim.x) counters[k] = 0;
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
                                                            int2* __restrict__ win, int* __restrict__ err,
                                                            int* __restrict__ widest,
                                                            const float* __restrict__ val = nullptr,
                                                            int* __restrict__ nonuniform = nullptr,
                                                            int nrows = -1) {  // rows of idx, if not N (VirtInfo layers)
    // The window is cyclic (see win_rel): two candidate cuts of the circle are tried, the row end and the
    // row's middle (columns shifted by h), and the narrower window wins.
    __shared__ int s_lo, s_hi, s_lo2, s_hi2;
    const int tid = threadIdx.x;
    const int j = blockIdx.x * kBlk + tid;
    const int h = (N / 2) & ~3;
    if (tid == 0) {
        s_lo = s_lo2 = N;
        s_hi = s_hi2 = -1;
    }
    __syncthreads();
    int lo = N, hi = -1, lo2 = N, hi2 = -1;
    if (j < (nrows < 0 ? N : nrows)) {
        for (int k = 0; k < kNnz; ++k) {
            const int c = idx[(size_t)j * kNnz + k];
            if (c < 0 || c >= N) {
                *err = 1;
            } else {
                lo = min(lo, c);
                hi = max(hi, c);
                const int c2 = c + h >= N ? c + h - N : c + h;
                lo2 = min(lo2, c2);
                hi2 = max(hi2, c2);
            }
        }
        if (val) {  // does the whole layer use one weight (bit for bit)?
            const uint32_t w0 = __builtin_bit_cast(uint32_t, val[0]);
            bool same = true;
            for (int k = 0; k < kNnz; ++k) same = same && __builtin_bit_cast(uint32_t, val[(size_t)j * kNnz + k]) == w0;
            if (!same) *nonuniform = 1;
        }
    }
    atomicMin(&s_lo, lo);
    atomicMax(&s_hi, hi);
    atomicMin(&s_lo2, lo2);
    atomicMax(&s_hi2, hi2);
    __syncthreads();
    if (tid == 0) {
        int c_lo = 0, ncols = 4;
        if (s_hi >= s_lo) {
            c_lo = s_lo & ~3;
            ncols = ((s_hi + 1 - c_lo) + 3) & ~3;
            const int c_lo2 = s_lo2 & ~3;
            const int ncols2 = ((s_hi2 + 1 - c_lo2) + 3) & ~3;
            if (ncols2 < ncols) {  // narrower when cut at the row's middle: back to unshifted columns
                ncols = ncols2;
                c_lo = c_lo2 - h < 0 ? c_lo2 - h + N : c_lo2 - h;
            }
        }
        win[blockIdx.x] = make_int2(c_lo, ncols);
        atomicMax(widest, ncols);  // the layer's widest window (zero before the launch)
    }
}

// ---------------------------------------------------------------------------
// a0 for general sparse layers (Section II-A-1: W_l may be any sparse matrix; Listing 1
// holds it in CSR; Section III-A-3 pads the neurons of a warp to a common length with
// zeros): neuron j owns entries ptr[j] .. ptr[j+1]-1.  A layer whose longest neuron
// has K connections is cut into ceil(K/32) passes of 32 connections per neuron, short
// neurons padded with zero weights, and every pass then goes through the set-up of a
// fixed-32 layer.
// ---------------------------------------------------------------------------
// out[0] = longest neuron (atomic max; zero before the launch), out[1] = 1 if ptr is
// negative somewhere or decreases.
__global__ void csr_scan_kernel(const int32_t* __restrict__ ptr, int N, int* __restrict__ out) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= N) return;
    const int a = ptr[j], e = ptr[j + 1];
    if (a < 0 || e < a)
        out[1] = 1;
    else
        atomicMax(out, e - a);
}

// Column window of every 1024-neuron block of a general layer, over all of its neurons'
// connections (valid columns only): win[b] = {first column, columns}, {0, 0} if it has none.
__global__ __launch_bounds__(kBlk) void csr_block_window_kernel(const int32_t* __restrict__ ptr,
                                                                const int32_t* __restrict__ idx, int N,
                                                                int2* __restrict__ win) {
    __shared__ int s_lo, s_hi;
    if (threadIdx.x == 0) {
        s_lo = N;
        s_hi = -1;
    }
    __syncthreads();
    const int j = blockIdx.x * kBlk + threadIdx.x;
    int lo = N, hi = -1;
    if (j < N) {
        const int a = ptr[j], e = ptr[j + 1];
        for (int k = a; k < e; ++k) {
            const int c = idx[k];
            if (c >= 0 && c < N) {
                lo = min(lo, c);
                hi = max(hi, c);
            }
        }
    }
    atomicMin(&s_lo, lo);
    atomicMax(&s_hi, hi);
    __syncthreads();
    if (threadIdx.x == 0) win[blockIdx.x] = s_hi >= s_lo ? make_int2(s_lo, s_hi + 1 - s_lo) : make_int2(0, 0);
}

// Pass r of a layer: smallest valid column among entries 32r .. 32r+31 of the neurons of
// every 1024-neuron block (blockmin[b] = N before the launch).  The padding points there,
// so that it does not widen the block's column window.
__global__ __launch_bounds__(kBlk) void csr_block_min_kernel(const int32_t* __restrict__ ptr,
                                                             const int32_t* __restrict__ idx, int N, int r,
                                                             int* __restrict__ blockmin) {
    __shared__ int s_lo;
    if (threadIdx.x == 0) s_lo = N;
    __syncthreads();
    const int j = blockIdx.x * kBlk + threadIdx.x;
    int lo = N;
    if (j < N) {
        const int a = ptr[j] + r * kNnz;
        const int e = min(ptr[j + 1], a + kNnz);
        for (int k = a; k < e; ++k) {
            const int c = idx[k];
            if (c >= 0) lo = min(lo, c);
        }
    }
    atomicMin(&s_lo, lo);
    __syncthreads();
    if (threadIdx.x == 0) blockmin[blockIdx.x] = s_lo;
}

// Pass r of a layer as a fixed-32 layer: out_idx / out_val [N][32].  One thread per entry.
__global__ void csr_round_kernel(const int32_t* __restrict__ ptr, const int32_t* __restrict__ idx,
                                 const float* __restrict__ val, int N, int r, const int* __restrict__ blockmin,
                                 int32_t* __restrict__ out_idx, float* __restrict__ out_val) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)N * kNnz) return;
    const int j = (int)(i / kNnz);
    const int k = (int)(i % kNnz);
    const int a = ptr[j] + r * kNnz + k;
    if (a < ptr[j + 1]) {
        out_idx[i] = idx[a];
        out_val[i] = val[a];
    } else {
        const int lo = blockmin[j / kBlk];
        out_idx[i] = lo < N ? lo : 0;
        out_val[i] = 0.0f;
    }
}

// Smallest and largest column of every four neighbouring neurons of a general layer ({N, -1}: no connection):
// what the host packs the workgroups of a several-lanes-per-neuron layer by.
__global__ void csr_quartet_window_kernel(const int32_t* __restrict__ ptr, const int32_t* __restrict__ idx, int N,
                                          int2* __restrict__ out) {
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (4 * q >= N) return;
    int lo = N, hi = -1;
    for (int e = ptr[4 * q]; e < ptr[4 * q + 4]; ++e) {
        const int c = idx[e];
        if (c >= 0 && c < N) {
            lo = min(lo, c);
            hi = max(hi, c);
        }
    }
    out[q] = make_int2(lo, hi);
}

// A general layer with several lanes per neuron (VirtInfo), as a fixed-32 layer of lanes.  Workgroup blockIdx.x
// has the neurons range[blockIdx.x].x .. + range[blockIdx.x].y - 1 (at most 1024 parts of 32 connections together,
// the host sees to that).  The parts are numbered neuron by neuron (that number is the part's slot) and ranked by
// length, longest first, equal lengths in slot order; the part of rank i becomes lane i: out_idx / out_val
// [.][32] hold its connections, padded with weight 0 on the workgroup's smallest column, len its length, slot
// its slot; fin[i] = first slot | number of slots << 16 of the workgroup's i-th neuron.
__global__ __launch_bounds__(kBlk) void csr_virtual_kernel(const int32_t* __restrict__ ptr,
                                                           const int32_t* __restrict__ idx,
                                                           const float* __restrict__ val, int N,
                                                           const int2* __restrict__ range,
                                                           int32_t* __restrict__ out_idx, float* __restrict__ out_val,
                                                           uint8_t* __restrict__ len, uint16_t* __restrict__ slot,
                                                           uint32_t* __restrict__ fin) {
    __shared__ uint8_t len_s[kBlk];
    __shared__ uint16_t part_neuron[kBlk], part_no[kBlk];
    __shared__ int wave_sum[17];
    __shared__ int s_lo;
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int2 rg = range[blockIdx.x];
    if (t == 0) s_lo = N;
    // parts of my neuron (thread i < rg.y has the workgroup's i-th neuron) and where they start
    const int jn = rg.x + t;
    const int parts = (t < rg.y && jn < N) ? (ptr[jn + 1] - ptr[jn] + kNnz - 1) / kNnz : 0;
    int incl = parts;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
    }
    if (lane == 63) wave_sum[wave] = incl;
    __syncthreads();
    if (t == 0) {
        int run = 0;
        for (int k = 0; k < 16; ++k) {
            const int v = wave_sum[k];
            wave_sum[k] = run;
            run += v;
        }
        wave_sum[16] = run;
    }
    __syncthreads();
    const int first_slot = wave_sum[wave] + incl - parts;
    const int total = min(wave_sum[16], kBlk);  // never more than 1024: the host packed the workgroups
    fin[(size_t)blockIdx.x * kBlk + t] = (uint32_t)first_slot | ((uint32_t)parts << 16);
    for (int p = 0; p < parts && first_slot + p < kBlk; ++p) {
        part_neuron[first_slot + p] = (uint16_t)t;
        part_no[first_slot + p] = (uint16_t)p;
    }
    __syncthreads();
    // thread t now is part (slot) t
    int first = 0, mine = 0;
    if (t < total) {
        const int j = rg.x + part_neuron[t];
        first = ptr[j] + (int)part_no[t] * kNnz;
        mine = max(0, min(kNnz, ptr[j + 1] - first));
    }
    int lo = N;
    for (int k = 0; k < mine; ++k) {
        const int c = idx[first + k];
        if (c >= 0) lo = min(lo, c);
    }
    atomicMin(&s_lo, lo);
    len_s[t] = (uint8_t)mine;
    __syncthreads();
    const int pad = s_lo < N ? s_lo : 0;
    int rank = 0;
    for (int o = 0; o < kBlk; ++o) {
        const int other = len_s[o];
        rank += (other > mine || (other == mine && o < t)) ? 1 : 0;
    }
    const size_t ln = (size_t)blockIdx.x * kBlk + rank;
    len[ln] = (uint8_t)mine;
    slot[ln] = (uint16_t)t;  // slots past `total` belong to lanes without connections; nobody adds them up
    for (int k = 0; k < kNnz; ++k) {
        out_idx[ln * kNnz + k] = k < mine ? idx[first + k] : pad;
        out_val[ln * kNnz + k] = k < mine ? val[first + k] : 0.0f;
    }
}

// Can the layer run two output neurons per lane?  Yes if all its weights are equal, N
// is a multiple of 2048 and either the windows of output blocks 2u and 2u+1 together
// span at most kCap columns for every u (info[0] = 1: fused_pair_kernel) or every block
// needs 2 or more stages anyway (info[0] = 2: the wide pair kernels, if the pattern fits
// the wide format).  Then both blocks of a unit get their common window.  info[0] = 0
// otherwise; info[1] = the weight's bits.  One workgroup.
__global__ __launch_bounds__(64) void pair_merge_kernel(int2* __restrict__ win, int nblk, int N,
                                                        const float* __restrict__ val,
                                                        const int* __restrict__ nonuniform,
                                                        int* __restrict__ widest, int* __restrict__ info) {
    __shared__ int s_max;
    const int t = threadIdx.x;
    if (t == 0) s_max = 0;
    __syncthreads();
    const bool candidate = *nonuniform == 0 && (N % (2 * kBlk)) == 0;
    if (candidate) {
        for (int u = t; u < nblk / 2; u += 64) {
            const int2 a = win[2 * u], c = win[2 * u + 1];
            int ux, uy;
            win_union(a.x, a.y, c.x, c.y, N, ux, uy);
            atomicMax(&s_max, uy);
        }
    }
    __syncthreads();
    // 1: one stage suffices for every unit; 2: every block needs 2 or more stages on its own
    // (the wide format, which also profits from common windows); otherwise hands off
    int s_min = 1 << 30;
    for (int bb = 0; bb < nblk; ++bb) s_min = min(s_min, win[bb].y);
    const int mode = !candidate ? 0 : s_max <= kCap ? 1 : s_min > kCap ? 2 : 0;
    const bool ok = mode != 0;
    __syncthreads();
    if (ok) {
        for (int u = t; u < nblk / 2; u += 64) {
            const int2 a = win[2 * u], c = win[2 * u + 1];
            int ux, uy;
            win_union(a.x, a.y, c.x, c.y, N, ux, uy);
            win[2 * u] = win[2 * u + 1] = make_int2(ux, uy);
        }
        if (t == 0) atomicMax(widest, s_max);
    }
    if (t == 0) {
        info[0] = mode;
        info[1] = __builtin_bit_cast(int, val[0]);
    }
}

// Balanced tile layout for single-stage layers (widest window <= kCap columns).
//
// The bank-aware ordering (spdnn_order.h) can only spread a lane set's 512
// connections over the 32 steps as evenly as they are spread over the 16 bank quads:
// the busiest quad's count is a lower bound on the set's cost.  With a fixed
// column -> quad rule that maximum is about 45 for random patterns (mean 32), i.e. 40 %
// more LDS read cycles than necessary.  Which quad a column's 16-byte entry sits in is,
// however, free inside its store group (see store_group()), so it is chosen here, per
// output block, to even out every set's quad histogram: the store groups are taken in
// turn; a column's cost for quad q is the sum, over its connections, of what q already
// holds for the connection's lane set; columns pick their cheapest free quad, busiest
// column first.  Measured on the 65536-neuron patterns: busiest quad 33.6 on average,
// 4.3 LDS cycles per 64-lane read instead of 5.7 (4 is conflict-free).
//
// One wave per output block.  Output: slot_tab[b][c] = LDS slot of stage-local column
// c, qsel[b][t] = quads (times 16, one per byte) of staging lane t's four columns.
// A layer with a wider window is left alone (order_pack_kernel then uses col_slot()).
// UB = output blocks per unit: 1, or 2 for layers that run two neurons per lane (the
// two blocks then share window, tile layout and staging quads, stored under the first).
template <int UB>
struct BalanceScratch {
    uint32_t cursor[kCap];                 // connections per column, then fill position
    uint32_t ofs[kCap + 4];                // start of column c's entries in ent[]
    uint8_t ent[UB * kNnz * kBlk];         // lane set (0..64*UB-1) of every connection, grouped by column
    uint32_t load[UB * kBlk / kGroup][16];  // connections lane set S already has in quad q
    uint16_t cost[16][16];
};
constexpr int kBalanceThreads = 64;
template <int UB>
__global__ __launch_bounds__(kBalanceThreads) void balance_kernel(const int32_t* __restrict__ idx, int N,
                                                                  const int2* __restrict__ win,
                                                                  const int* __restrict__ widest,
                                                                  uint16_t* __restrict__ slot_tab,
                                                                  uint32_t* __restrict__ qsel,
                                                                  int nrows = -1) {  // rows of idx, if not N
    extern __shared__ __align__(16) char balance_scratch[];
    BalanceScratch<UB>& B = *reinterpret_cast<BalanceScratch<UB>*>(balance_scratch);
    if (*widest > kCap) return;
    const int b = blockIdx.x * UB;
    const int lane = threadIdx.x;
    const int c_lo = win[b].x;
    for (int c = lane; c < kCap; c += kBalanceThreads) B.cursor[c] = 0;
    for (int i = lane; i < UB * (kBlk / kGroup) * 16; i += kBalanceThreads) (&B.load[0][0])[i] = 0;
    __syncthreads();
    // stage-local column of connection e = (neuron << 5 | k) of this unit, or -1
    auto rel_of = [&](int e) -> int {
        const int j = b * kBlk + (e >> 5);
        if (j >= (nrows < 0 ? N : nrows)) return -1;
        const int c = idx[(size_t)j * kNnz + (e & 31)];
        return (c < 0 || c >= N) ? 0 : win_rel(c, c_lo, N);  // out-of-range columns were reported; keep them harmless
    };
    for (int e = lane; e < UB * kNnz * kBlk; e += kBalanceThreads) {
        const int r = rel_of(e);
        if (r >= 0) atomicAdd(&B.cursor[r], 1u);
    }
    __syncthreads();
    // exclusive prefix sum over the columns: lane owns 64 consecutive ones
    {
        constexpr int per = kCap / kBalanceThreads;
        uint32_t sum = 0;
        for (int i = 0; i < per; ++i) sum += B.cursor[lane * per + i];
        uint32_t incl = sum;
        for (int d = 1; d < kBalanceThreads; d <<= 1) {
            const uint32_t v = __shfl_up(incl, d);
            if (lane >= d) incl += v;
        }
        uint32_t run = incl - sum;
        for (int i = 0; i < per; ++i) {
            const uint32_t n = B.cursor[lane * per + i];
            B.ofs[lane * per + i] = run;
            B.cursor[lane * per + i] = run;
            run += n;
        }
        if (lane == kBalanceThreads - 1) B.ofs[kCap] = run;
    }
    __syncthreads();
    for (int e = lane; e < UB * kNnz * kBlk; e += kBalanceThreads) {
        const int r = rel_of(e);
        if (r < 0) continue;
        const uint32_t pos = atomicAdd(&B.cursor[r], 1u);
        const uint32_t n = (uint32_t)e >> 5;
        B.ent[pos] = (uint8_t)(((n >> 6) << 2) | set_of_lane(n & 63u));
    }
    __syncthreads();

    // Cost phase: lanes 4 i .. 4 i + 3 share column i of the group, each takes every fourth of its connections
    // and adds up, for all 16 quads, what the connections' lane sets already hold there.
    const int row = lane >> 2;
    const int sub = lane & 3;
    uint32_t packed = 0;  // lanes 0..15: quads (times 16) chosen so far for the staging lane's columns
    for (int g = 0; g < kCap / 16; ++g) {
        const int a = g & 3, set = (g >> 2) & 3, wave = g >> 4;
        auto column_of = [&](int i) { return 4 * (wave * 64 + lane_of_group(set, i)) + a; };
        const int c_row = column_of(row);
        const uint32_t e0 = B.ofs[c_row], e1 = B.ofs[c_row + 1];
        // The columns choose in the order of their connection counts, busiest first, lowest index among equals:
        // known before any cost is.  rank = my column's place in that order (every 16 lanes: column lane & 15).
        const int c_mine = column_of(lane & 15);
        const int cnt = (int)B.ofs[c_mine + 1] - (int)B.ofs[c_mine];
        int rank = 0;
        {
            const int key = (cnt << 4) | (15 - (lane & 15));
#define SPDNN_RANK_STEP(n) rank += __builtin_amdgcn_mov_dpp(key, 0x120 + (n), 0xF, 0xF, true) > key ? 1 : 0;
            SPDNN_RANK_STEP(1) SPDNN_RANK_STEP(2) SPDNN_RANK_STEP(3) SPDNN_RANK_STEP(4) SPDNN_RANK_STEP(5)
            SPDNN_RANK_STEP(6) SPDNN_RANK_STEP(7) SPDNN_RANK_STEP(8) SPDNN_RANK_STEP(9) SPDNN_RANK_STEP(10)
            SPDNN_RANK_STEP(11) SPDNN_RANK_STEP(12) SPDNN_RANK_STEP(13) SPDNN_RANK_STEP(14) SPDNN_RANK_STEP(15)
#undef SPDNN_RANK_STEP
        }
        const int rank_row = __shfl(rank, row);  // of column `row`: its costs go to row rank_row of the table
        {
            uint32_t acc[16];
#pragma unroll
            for (int q = 0; q < 16; ++q) acc[q] = 0;
            for (uint32_t e = e0 + sub; e < e1; e += 4) {
                const uint4* ld = reinterpret_cast<const uint4*>(&B.load[B.ent[e]][0]);
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const uint4 x = ld[v];
                    acc[4 * v + 0] += x.x;
                    acc[4 * v + 1] += x.y;
                    acc[4 * v + 2] += x.z;
                    acc[4 * v + 3] += x.w;
                }
            }
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                acc[q] += (uint32_t)__builtin_amdgcn_mov_dpp((int)acc[q], 0xB1, 0xF, 0xF, true);  // lanes ^ 1
                acc[q] += (uint32_t)__builtin_amdgcn_mov_dpp((int)acc[q], 0x4E, 0xF, 0xF, true);  // lanes ^ 2
            }
            if (sub == 0) {
                uint32_t* out = reinterpret_cast<uint32_t*>(&B.cost[rank_row][0]);
#pragma unroll
                for (int q = 0; q < 16; q += 2) out[q >> 1] = min(acc[q], 4095u) | (min(acc[q + 1], 4095u) << 16);
            }
        }
        __syncthreads();
        // every 16 lanes in two roles: as column i = lane & 15 (chosen quad) and as quad q = lane & 15; the costs
        // of the 16 turns are fetched at once, the turns themselves are a reduction each
        int cst[16];
#pragma unroll
        for (int it = 0; it < 16; ++it) cst[it] = (int)B.cost[it][lane & 15];
        int chosen = -1;
        bool quad_free = true;
#pragma unroll
        for (int it = 0; it < 16; ++it) {  // the column of rank `it` picks its cheapest free quad, the lowest among equals
            const int k2 = quad_free ? ((cst[it] << 4) | (lane & 15)) : 0x7fffffff;
            const int q = row16_min(k2) & 15;
            if (rank == it) chosen = q;
            if ((lane & 15) == q) quad_free = false;
        }
        // the chosen quads take the columns' connections on board (all 64 lanes: column `row`, every fourth entry)
        {
            const int ch = __shfl(chosen, row);
            for (uint32_t e = e0 + sub; e < e1; e += 4) atomicAdd(&B.load[B.ent[e]][ch], 1u);
        }
        if (lane < 16) {
            slot_tab[(size_t)b * kCap + c_mine] = (uint16_t)((g << 4) | chosen);
            packed |= (uint32_t)(chosen << 4) << (8 * a);
            if (a == 3) {
                qsel[(size_t)b * kBlk + wave * 64 + lane_of_group(set, lane)] = packed;
                packed = 0;
            }
        }
        __syncthreads();
    }
}

// One wave per set of 16 neurons whose lanes are served together: orders the set's
// connections for conflict-free LDS reads and writes them lane-major: entry
// (block b, step s, lane t) holds the LDS slot of the connection's column (plus
// the stage number in bits 12 and up) and its weight, for the connection lane t
// uses at step s.
//
// The ordering is order_group's (spdnn_order.h), choice for choice, with the wave's first 16 lanes in
// two roles: lane l as the set's l-th neuron (its unplaced connections, its quad of the current step,
// its parent in the search) and lane q as bank quad q (the lanes that still have a connection there,
// how many connections, how many lanes use it in this step).  What the serial routine loops over is a
// 16-lane reduction or a bit mask here; the breadth-first search stays serial, one quad per turn.
// A thread per set took 3.1 ms per 65536-neuron layer.
constexpr int kOrderThreads = kBlk / kGroup;  // lane sets per output block
constexpr int kOrderPackThreads = 64;
struct Pack16Scratch {
    uint32_t conn[16][16];  // [q][l]: connections (bit k) of lane l that fall in quad q
    uint32_t adj[16];       // lanes that still have a connection in quad q
    uint32_t remq[16];      // connections not placed yet in quad q, whole set
    uint32_t queue[20];
};
__global__ __launch_bounds__(kOrderPackThreads) void order_pack_kernel(const int32_t* __restrict__ idx,
                                                                   const float* __restrict__ val, int N,
                                                                   const int2* __restrict__ win,
                                                                   const int* __restrict__ widest,
                                                                   const uint16_t* __restrict__ slot_tab,
                                                                   int pair,  // the layer's tile layout is per two blocks
                                                                   uint16_t* __restrict__ rel,
                                                                   float* __restrict__ wval,
                                                                   // VirtInfo layers: idx / val have nrows rows (all of them
                                                                   // lanes that exist), row i holds len[i] connections, and
                                                                   // a set's connections are placed in the first steps only,
                                                                   // as many (in eights) as its longest lane needs;
                                                                   // nb8[block][wave] = blocks of 8 steps the wave then runs
                                                                   int nrows = -1, const uint8_t* __restrict__ len = nullptr,
                                                                   uint8_t* __restrict__ nb8 = nullptr) {
    __shared__ Pack16Scratch S;
    const int gset = blockIdx.x;  // lane set, counted over the whole layer
    const int b = gset / kOrderThreads;
    const int t = gset - b * kOrderThreads;
    const int wave0 = (t >> 2) * 64;  // first lane of this set's wave inside the block
    const int set = t & 3;
    const int c_lo = win[b].x;
    const int rows = nrows < 0 ? N : nrows;
    const int lane = threadIdx.x;
    const bool on = lane < kGroup;  // the other lanes only keep the reductions company (and help with nb8)
    const int l = lane & 15;
    const int my_lane = wave0 + lane_of_group(set, l);  // my neuron's lane inside the block
    const int j = b * kBlk + my_lane;                   // my neuron
    const bool exists = j < rows;
    // LDS slot of stage-local column r: from balance_kernel for single-stage layers
    const bool balanced = *widest <= kCap;
    const uint16_t* tab = slot_tab + (size_t)(pair ? (b & ~1) : b) * kCap;
    auto slot_of = [&](uint32_t r) -> uint32_t { return balanced ? tab[r] : col_slot(r); };
    auto entry = [&](int step) -> size_t { return ((size_t)b * kNnz + step) * kBlk + my_lane; };
    int nsteps = kNnz;
    const int my_len = !exists ? 0 : len ? (int)len[j] : kNnz;
    if (len) {  // steps this set needs; everything else is weight 0 on the window's first column
        nsteps = (__builtin_amdgcn_readfirstlane(row16_max(on ? my_len : 0)) + 7) & ~7;
        const int jw = b * kBlk + wave0 + lane;  // lane `lane` of the wave this set belongs to
        int longest = jw < rows ? (int)len[jw] : 0;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) longest = max(longest, __shfl_xor(longest, d, 64));
        if (set == 0 && lane == 0 && nb8) nb8[b * 16 + (t >> 2)] = (uint8_t)(((longest + 7) & ~7) / 8);
    }
    if (on && (len || !exists)) {  // lanes past the last neuron, and the steps a short lane leaves empty
        const uint16_t zero_slot = (uint16_t)slot_of(0);
        for (int step = 0; step < kNnz; ++step) {
            rel[entry(step)] = zero_slot;
            wval[entry(step)] = 0.0f;
        }
    }
    auto column = [&](int k) -> int {  // out-of-range columns were reported; keep them harmless
        const int c = idx[(size_t)j * kNnz + k];
        return (c < 0 || c >= N) ? c_lo : c;
    };
    for (int q = 0; q < 16; ++q)
        if (on) S.conn[q][l] = 0;
    if (on) {
        S.adj[l] = 0;
        S.remq[l] = 0;
    }
    __syncthreads();
    uint32_t unplaced = 0;  // my connections not placed yet (bit k)
    if (on)
        for (int k = 0; k < my_len; ++k) {
            const int q = (int)(slot_of((uint32_t)win_rel(column(k), c_lo, N) & (kCap - 1)) & 15u);
            S.conn[q][l] |= 1u << k;  // my own column of the table
            unplaced |= 1u << k;
        }
    __syncthreads();
    if (on)
        for (int q = 0; q < 16; ++q) {
            const uint32_t m = S.conn[q][l];
            if (m) {
                atomicOr(&S.adj[q], 1u << l);
                atomicAdd(&S.remq[q], (uint32_t)__popc(m));
            }
        }
    __syncthreads();
    for (int step = 0; step < nsteps; ++step) {
        const int left = nsteps - step;
        const uint32_t adj = on ? S.adj[l] : 0u;  // as quad q = l
        const int remq = on ? (int)S.remq[l] : 0;
        int lane_of_quad = -1;  // as quad
        int quad_of_lane = -1;  // as lane
        int parent = -1;        // as lane: the quad from which the search reached me
        uint32_t free_lanes = 0xFFFFu;  // lanes without a quad (the same in every lane)
        uint32_t done = 0;              // quads already offered
        for (int r = 0; r < 16; ++r) {
            // the most urgent quad not offered yet, the lowest-numbered one among equals
            const int key = (!on || ((done >> l) & 1u)) ? -1 : ((((remq >= left) ? 4096 : 0) + remq) << 4) | (15 - l);
            const int best = __builtin_amdgcn_readfirstlane(row16_max(key));
            const int q0 = 15 - (best & 15);
            done |= 1u << q0;
            if (((best >> 4) & 4095) == 0) break;  // the rest are empty too
            // breadth-first search for an augmenting path from q0 to a free lane
            int head = 0, tail = 1, found = -1;
            uint32_t seen = 0;
            if (lane == 0) S.queue[0] = (uint32_t)q0;
            __syncthreads();
            while (head < tail && found < 0) {
                const int q = __builtin_amdgcn_readfirstlane((int)S.queue[head]);
                ++head;
                const uint32_t cand = (uint32_t)__builtin_amdgcn_readlane((int)adj, q) & ~seen;
                const uint32_t hit = cand & free_lanes;
                if (hit) {
                    found = __builtin_ctz(hit);
                    if (lane == found) parent = q;
                } else if (cand) {
                    seen |= cand;
                    if (on && ((cand >> l) & 1u)) {
                        parent = q;
                        S.queue[tail + __popc(cand & ((1u << l) - 1u))] = (uint32_t)quad_of_lane;  // a lane is seen once: at most 16 entries follow q0
                    }
                    tail += __popc(cand);
                    __syncthreads();
                }
            }
            if (found < 0) continue;
            free_lanes &= ~(1u << found);
            for (int cur = found;;) {
                const int q = __builtin_amdgcn_readlane(parent, cur);
                const int next = __builtin_amdgcn_readlane(lane_of_quad, q);  // meaningful only if q was matched
                if (lane == q) lane_of_quad = cur;
                if (lane == cur) quad_of_lane = q;
                if (q == q0) break;
                cur = next;
            }
        }
        // lanes without a quad of their own share the least loaded one they can use, in ascending order; a lane
        // with fewer connections left than steps sits this step out
        int mult = (on && lane_of_quad >= 0) ? 1 : 0;  // as quad: uses in this step (saturates at 15)
        const int reml = __popc(unplaced);
        for (uint32_t rest = free_lanes; rest;) {
            const int ll = __builtin_ctz(rest);
            rest &= rest - 1;
            const int r_ll = __builtin_amdgcn_readlane(reml, ll);
            if (r_ll == 0 || r_ll < left) continue;
            const uint32_t u_ll = (uint32_t)__builtin_amdgcn_readlane((int)unplaced, ll);
            const int cnt = on ? __popc(S.conn[l][ll] & u_ll) : 0;  // lane ll's unplaced connections in quad l
            const int key = cnt ? ((mult * 65536 - (remq - left) * 64 - cnt + 65536) << 4) | l : 0x7fffffff;
            const int bq = __builtin_amdgcn_readfirstlane(row16_min(key)) & 15;
            if (lane == ll) quad_of_lane = bq;
            if (lane == bq) mult = min(mult + 1, 15);
        }
        // place the chosen connections: the lowest unplaced one of the lane's quad
        if (on && quad_of_lane >= 0) {
            const uint32_t in_quad = S.conn[quad_of_lane][l];
            const int k = __builtin_ctz(in_quad & unplaced);
            unplaced &= ~(1u << k);
            atomicSub(&S.remq[quad_of_lane], 1u);
            if ((in_quad & unplaced) == 0) atomicAnd(&S.adj[quad_of_lane], ~(1u << l));
            const size_t src = (size_t)j * kNnz + k;
            const int c = idx[src];
            const bool ok = c >= 0 && c < N;
            const uint32_t r = ok ? (uint32_t)win_rel(c, c_lo, N) : 0u;  // stage number | slot inside the stage
            rel[entry(step)] = (uint16_t)((r & ~(uint32_t)(kCap - 1)) | slot_of(r & (kCap - 1)));
            wval[entry(step)] = ok ? val[src] : 0.0f;
        }
        __syncthreads();
    }
}

// Set-up of a wide layer (see WideWeights).  One thread per lane set, as in
// order_pack_kernel; phase 1 counts each lane's connections per stage and finds, per
// wave, how many blocks of 8 steps every stage needs; phase 2 orders each stage's
// connections over those steps and writes them out, unfilled steps with weight 0.
// *fail is set if some neuron would need more than kSpill spilled connections.
struct WideScratch {
    OrderScratch order;
    uint32_t keep[kGroup];  // per lane: connections placed in the current stage (bit k)
};
__global__ __launch_bounds__(kOrderThreads) void wide_pack_kernel(const int32_t* __restrict__ idx,
                                                                  const float* __restrict__ val, int N,
                                                                  const int2* __restrict__ win, int nstage,
                                                                  uint2* __restrict__ pk,
                                                                  uint8_t* __restrict__ nb8,
                                                                  uint16_t* __restrict__ spill_col,
                                                                  float* __restrict__ spill_val,
                                                                  uint8_t* __restrict__ spill_n,
                                                                  int* __restrict__ fail) {
    extern __shared__ WideScratch wide_scratch[];
    __shared__ int wave_need[16][16];  // [stage][wave] largest kept count
    __shared__ int wave_spill[16];
    const int S = wide_steps(nstage);
    const int b = blockIdx.x;
    const int t = threadIdx.x;
    const int wave = t >> 2;
    const int wave0 = wave * 64;
    const int set = t & 3;
    const int c_lo = win[b].x;
    for (int i = t; i < 16 * 16; i += kOrderThreads) (&wave_need[0][0])[i] = 0;
    if (t < 16) wave_spill[t] = 0;
    __syncthreads();
    auto neuron = [&](int l) -> int { return b * kBlk + wave0 + lane_of_group(set, l); };
    auto rel_of = [&](int l, int k) -> int {  // column relative to the window; bad columns were reported
        const int c = idx[(size_t)neuron(l) * kNnz + k];
        return (c < 0 || c >= N) ? 0 : win_rel(c, c_lo, N);
    };
    // phase 1: counts, spills
    for (int l = 0; l < kGroup; ++l) {
        const int j = neuron(l);
        const int lane_pos = wave0 + lane_of_group(set, l);
        int nsp = 0;
        if (j < N) {
            uint8_t cnt[16];
            for (int s = 0; s < 16; ++s) cnt[s] = 0;
            for (int k = 0; k < kNnz; ++k) {
                const int r = rel_of(l, k);
                const int s = r >> kCapLog2;
                if (cnt[s] < S) {
                    cnt[s]++;
                } else if (nsp < kSpill) {
                    const size_t se = ((size_t)b * kSpill + nsp) * kBlk + lane_pos;
                    const int c = idx[(size_t)j * kNnz + k];
                    spill_col[se] = (uint16_t)r;
                    spill_val[se] = (c < 0 || c >= N) ? 0.0f : val[(size_t)j * kNnz + k];
                    nsp++;
                } else {
                    *fail = 1;
                }
            }
            for (int s = 0; s < nstage; ++s) atomicMax(&wave_need[s][wave], (int)cnt[s]);
        }
        for (int e = nsp; e < kSpill; ++e) {
            const size_t se = ((size_t)b * kSpill + e) * kBlk + lane_pos;
            spill_col[se] = 0;
            spill_val[se] = 0.0f;
        }
        atomicMax(&wave_spill[wave], nsp);
    }
    __syncthreads();
    if (t < 16) spill_n[b * 16 + t] = (uint8_t)wave_spill[t];
    for (int i = t; i < nstage * 16; i += kOrderThreads)
        nb8[(size_t)b * nstage * 16 + i] = (uint8_t)((wave_need[i >> 4][i & 15] + 7) >> 3);
    // phase 2: per stage, order and write
    WideScratch& W = wide_scratch[t];
    for (int s = 0; s < nstage; ++s) {
        const int nsteps = ((wave_need[s][wave] + 7) >> 3) << 3;
        const size_t sbase = ((size_t)(b * nstage + s) * (S / 2)) * kBlk;  // in pairs of steps
        auto entry = [&](int step, int lane_pos) -> size_t {
            return ((sbase + (size_t)(step >> 1) * kBlk + lane_pos) << 1) | (size_t)(step & 1);
        };
        for (int l = 0; l < kGroup; ++l) {  // every step starts as "weight 0 on the stage's first column"
            const int lane_pos = wave0 + lane_of_group(set, l);
            for (int k = 0; k < S; ++k) pk[entry(k, lane_pos)] = make_uint2(col_slot(0), 0u);
            uint32_t keep = 0;
            if (neuron(l) < N) {
                int c = 0;
                for (int k = 0; k < kNnz; ++k)
                    if ((rel_of(l, k) >> kCapLog2) == s && c < S) {
                        keep |= 1u << k;
                        c++;
                    }
            }
            W.keep[l] = keep;
        }
        if (nsteps == 0) continue;
        uint16_t quads_of_step[32];  // bank quads the set's real reads use at each step
        uint32_t steps_of_lane[kGroup];
        for (int i = 0; i < 32; ++i) quads_of_step[i] = 0;
        for (int l = 0; l < kGroup; ++l) steps_of_lane[l] = 0;
        order_group(
            W.order, nsteps,
            [&](int l, int k) -> unsigned {
                return ((W.keep[l] >> k) & 1u) ? (col_slot((uint32_t)rel_of(l, k) & (kCap - 1)) & 15u) : 255u;
            },
            [&](int l, int step, int k) {
                const size_t src = (size_t)neuron(l) * kNnz + k;
                const int c = idx[src];
                const bool ok = c >= 0 && c < N;
                const uint32_t slot = col_slot((uint32_t)(ok ? win_rel(c, c_lo, N) : 0) & (kCap - 1));
                pk[entry(step, wave0 + lane_of_group(set, l))] =
                    make_uint2(slot, __builtin_bit_cast(uint32_t, ok ? val[src] : 0.0f));
                quads_of_step[step] |= (uint16_t)(1u << (slot & 15u));
                steps_of_lane[l] |= 1u << step;
            });
        // Steps a lane does not fill carry weight 0.  The lanes of a set are served in the same clock, so
        // the padding of a step reads from a quad that none of the set's real reads of that step uses
        // (there is one whenever there is padding); lanes that read the same entry do not collide.
        for (int step = 0; step < nsteps; ++step) {
            const uint32_t free_quads = ~(uint32_t)quads_of_step[step] & 0xFFFFu;
            const uint32_t q = free_quads ? (uint32_t)__builtin_ctz(free_quads) : 15u;
            for (int l = 0; l < kGroup; ++l)
                if (!((steps_of_lane[l] >> step) & 1u))
                    pk[entry(step, wave0 + lane_of_group(set, l))] = make_uint2(q, 0u);  // slot q lies in quad q
        }
    }
}

}  // namespace spdnn
