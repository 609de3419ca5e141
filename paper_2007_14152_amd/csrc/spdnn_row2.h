// a1 for layers whose blocks read (nearly) whole feature rows, with one weight for the whole
// layer: two rows per LDS entry, four output neurons per lane.
//
// A uniform pattern at N = 16384 makes every block of output neurons read the whole row, so
// what a workgroup stages is the row, whatever neurons it owns, and the bytes the CUs pull out
// of L2 are (row bytes) x (workgroups per row).  This kernel makes the workgroup as large as
// the register file allows -- 4096 neurons, four per lane, their 32 LDS addresses packed two
// per register (64 registers) -- so a row is staged by N / 4096 workgroups.  The tile is the
// whole column window (up to 16384 columns) of TWO rows, 8 bytes per column (128 KB of LDS):
// every connection is one ds_read_b64 feeding two FMAs, a neuron takes exactly its 32 steps
// (no stages, hence no padding steps), and the sum runs in the order the set-up chose for the
// LDS banks (row2_pack_kernel), one fused multiply-add per connection, bias last.
//
// One tile fills the LDS, so there is one buffer: the next tile waits in registers and is written
// between two barriers once every wave is done reading; that write phase is not hidden (about a
// sixth of a step).  The loads of the next tile are issued in four bursts spread over the compute
// phase, as instructions with a scalar base (no vector registers for addresses; the wait for them is
// written out by hand).  The staged values must never be spilled between a load and that wait --
// the compiler does not know they arrive late -- so the build checks that this kernel uses no
// scratch memory.
#pragma once

namespace spdnn {

constexpr int kRows2 = 2;            // feature rows per tile
constexpr int kUnit4 = 4 * kBlk;     // output neurons per workgroup
constexpr int kRow2Cols = 16384;     // columns a tile holds
constexpr int kRow2Bursts = 4;       // bursts in which a tile's eight loads per lane are issued (2, 4 or 8; measured: 4)
constexpr int kRow2Seg = 4096;       // columns staged per lane and segment (1024 lanes x 4 columns)
constexpr int kRow2TileBytes = kRow2Cols * kRows2 * 4;
constexpr int kRow2LdsBytes = kRow2TileBytes + kUnit4 * 4;  // the tile, then the unit's biases

struct Row2Weights {
    const uint4* codes;  // [nunit][4][4][kBlk]: neuron slot s of lane t, steps 8o .. 8o+7 as 16-bit tile positions
                         // (row2_pos of the column inside the unit's window)
    const int2* win;     // [nblk] per 1024-neuron block {c_lo, ncols}; a unit's window is the union of its four
    const int32_t* map;  // NULL: the tile is the unit's contiguous window.  Else the gathered footprint (the preload
                         // list of Section III-A-2, at 4-column granularity): [nunit][4096] first column of the
                         // group of four columns that tile slot g holds (row2_gather_kernel says in which order);
                         // slots without a group repeat the unit's last.  Tile column 4g + a is row column map[g] + a.
    int seg_log2;        // the unit's neurons: 4096 >> seg_log2 segments of 1 << seg_log2 neighbours, one every
    int seg_stride;      // seg_stride neurons (unit_neuron); 12 = one run of 4096 (then seg_stride is not used)
};

// Column window of unit u: the union of its four blocks' (cyclic) windows; c_lo a multiple of 4.
__device__ __forceinline__ int2 row2_window(const int2* __restrict__ win, int u, int N) {
    int x = 0, y = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int2 w = win[4 * u + i];
        win_union(x, y, w.x, w.y, N, x, y);
    }
    return make_int2(x, y);
}

// 16 connections of one neuron: acc[r] = fma(tile[col_k][r], w, acc[r]), k = 0..15 in that order.
// p[i] holds the (LDS byte address >> 3) of connections 2i and 2i+1 in its halves; an SDWA shift
// turns a half into the byte address, written into the first register of the read's own
// destination; s3 (scalar) holds 3.  Two reads in flight in v124..v127 (with 16 waves per CU the LDS
// stays busy at this depth, and the kernel needs every other register).
__device__ __forceinline__ void fma_row2_block16(float (&acc)[kRows2], const uint32_t* p, float w, uint32_t s3) {
    asm volatile(
        "v_lshlrev_b32_sdwa v120, %[s3], %[p0] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
        "ds_read_b64 v[120:121], v120\n\t"
        "v_lshlrev_b32_sdwa v122, %[s3], %[p0] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n\t"
        "ds_read_b64 v[122:123], v122\n\t"
        "v_lshlrev_b32_sdwa v124, %[s3], %[p1] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
        "ds_read_b64 v[124:125], v124\n\t"
        "v_lshlrev_b32_sdwa v126, %[s3], %[p1] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n\t"
        "ds_read_b64 v[126:127], v126\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v120\n\t"
        "v_fmac_f32 %[a1], %[w], v121\n\t"
        "v_lshlrev_b32_sdwa v120, %[s3], %[p2] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
        "ds_read_b64 v[120:121], v120\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v122\n\t"
        "v_fmac_f32 %[a1], %[w], v123\n\t"
        "v_lshlrev_b32_sdwa v122, %[s3], %[p2] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n\t"
        "ds_read_b64 v[122:123], v122\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v124\n\t"
        "v_fmac_f32 %[a1], %[w], v125\n\t"
        "v_lshlrev_b32_sdwa v124, %[s3], %[p3] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
        "ds_read_b64 v[124:125], v124\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v126\n\t"
        "v_fmac_f32 %[a1], %[w], v127\n\t"
        "v_lshlrev_b32_sdwa v126, %[s3], %[p3] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n\t"
        "ds_read_b64 v[126:127], v126\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v120\n\t"
        "v_fmac_f32 %[a1], %[w], v121\n\t"
        "v_lshlrev_b32_sdwa v120, %[s3], %[p4] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
        "ds_read_b64 v[120:121], v120\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v122\n\t"
        "v_fmac_f32 %[a1], %[w], v123\n\t"
        "v_lshlrev_b32_sdwa v122, %[s3], %[p4] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n\t"
        "ds_read_b64 v[122:123], v122\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v124\n\t"
        "v_fmac_f32 %[a1], %[w], v125\n\t"
        "v_lshlrev_b32_sdwa v124, %[s3], %[p5] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
        "ds_read_b64 v[124:125], v124\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v126\n\t"
        "v_fmac_f32 %[a1], %[w], v127\n\t"
        "v_lshlrev_b32_sdwa v126, %[s3], %[p5] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n\t"
        "ds_read_b64 v[126:127], v126\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v120\n\t"
        "v_fmac_f32 %[a1], %[w], v121\n\t"
        "v_lshlrev_b32_sdwa v120, %[s3], %[p6] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
        "ds_read_b64 v[120:121], v120\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v122\n\t"
        "v_fmac_f32 %[a1], %[w], v123\n\t"
        "v_lshlrev_b32_sdwa v122, %[s3], %[p6] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n\t"
        "ds_read_b64 v[122:123], v122\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v124\n\t"
        "v_fmac_f32 %[a1], %[w], v125\n\t"
        "v_lshlrev_b32_sdwa v124, %[s3], %[p7] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
        "ds_read_b64 v[124:125], v124\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v126\n\t"
        "v_fmac_f32 %[a1], %[w], v127\n\t"
        "v_lshlrev_b32_sdwa v126, %[s3], %[p7] dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1\n\t"
        "ds_read_b64 v[126:127], v126\n\t"
        "s_waitcnt lgkmcnt(3)\n\t"
        "v_fmac_f32 %[a0], %[w], v120\n\t"
        "v_fmac_f32 %[a1], %[w], v121\n\t"
        "s_waitcnt lgkmcnt(2)\n\t"
        "v_fmac_f32 %[a0], %[w], v122\n\t"
        "v_fmac_f32 %[a1], %[w], v123\n\t"
        "s_waitcnt lgkmcnt(1)\n\t"
        "v_fmac_f32 %[a0], %[w], v124\n\t"
        "v_fmac_f32 %[a1], %[w], v125\n\t"
        "s_waitcnt lgkmcnt(0)\n\t"
        "v_fmac_f32 %[a0], %[w], v126\n\t"
        "v_fmac_f32 %[a1], %[w], v127\n\t"
        : [a0] "+v"(acc[0]), [a1] "+v"(acc[1])
        : [p0] "v"(p[0]), [p1] "v"(p[1]), [p2] "v"(p[2]), [p3] "v"(p[3]), [p4] "v"(p[4]), [p5] "v"(p[5]), [p6] "v"(p[6]),
          [p7] "v"(p[7]), [w] "s"(w), [s3] "s"(s3)
        : "v120", "v121", "v122", "v123", "v124", "v125", "v126", "v127", "memory");
}

__global__ __launch_bounds__(kBlk) void fused_row2_kernel(
    const float* __restrict__ Yin, float* __restrict__ Yout, uint8_t* __restrict__ flags,
    RowLists rl, Row2Weights w,
    const float* __restrict__ bias, int N, int nunit, int G, int Q, float wuni) {
    extern __shared__ float4 lds4[];
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    using lds_f2 = __attribute__((address_space(3))) f32x2;
    const int tid = threadIdx.x;
    const int lane = tid & 63;

    WorkItem wi;  // my unit and my groups of two rows
    __shared__ int rl_red[17], rl_scan[17];
    if (!derive_work(rl, nunit, G, Q, wi, kRows2, rl_red, rl_scan)) return;
    const int* cat = rl.cat;      // my slice of it was written just now
    const int u = wi.cb, A = wi.A, g0 = wi.g0, g1 = wi.g1;
    const bool gathered = w.map != nullptr;  // the tile is a gathered list of 4-column groups, not a window
    const int2 win = gathered ? make_int2(0, kRow2Cols) : row2_window(w.win, u, N);
    const int c_lo = win.x;
    const int ncols = win.y;  // <= kRow2Cols, a multiple of 4
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds4;
    uint32_t s3 = 3;
    asm volatile("" : "+s"(s3));  // the shift count of fma_row2_block32, kept in a scalar register

    // step lists of my four neurons (u * 4096 + s * 1024 + tid), two LDS addresses (>> 3) per register
    uint32_t p[4][16];
    {
        const uint32_t base8 = lds_base >> 3;
        const uint32_t both = base8 | (base8 << 16);
        const uint4* q = w.codes + (size_t)u * 16 * kBlk + tid;
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int o = 0; o < 4; ++o) {
                const uint4 v = q[(s * 4 + o) * kBlk];
                p[s][o * 4 + 0] = v.x + both;
                p[s][o * 4 + 1] = v.y + both;
                p[s][o * 4 + 2] = v.z + both;
                p[s][o * 4 + 3] = v.w + both;
            }
    }

    // Staging.  Lane t owns columns 4t .. 4t+3 of each 4096-column segment of the window: one
    // 16-byte load per row and segment, one 8-byte LDS entry (the two rows of a column) per column.
    // Addresses are a scalar row base plus a 32-bit lane offset.
    const int nseg = (ncols + kRow2Seg - 1) / kRow2Seg;
    f32x4 st[4][kRows2];
    const uint32_t st_addr = lds_base + 8u * (((4u * tid) & ~127u) | (tid & 31u));  // entry of column 4t; +256 per column
    ListWindow rows_of(cat, g0 * kRows2, min(A, g1 * kRows2), wi.identity);
    const int cat_last = rows_of.last();  // used by the last, ragged group only: then the list's last entry
    const int T = g1 - g0;
    // Byte offset, from the start of a row, of my four columns in every segment.  In a narrower last segment
    // the lanes past the window re-read its last columns; the window is cyclic (it may run over the row end);
    // with a gathered footprint the offsets come from the unit's list.
    const int last_cols = ncols - (nseg - 1) * kRow2Seg;  // columns of the last segment (a multiple of 4, >= 4)
    uint32_t off[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int rel = s * kRow2Seg + (s == nseg - 1 ? min(4 * tid, last_cols - 4) : 4 * tid);
        off[s] = 4u * (uint32_t)win_col(c_lo, min(rel, ncols - 4), N);
        if (gathered) off[s] = 4u * (uint32_t)w.map[(size_t)u * (kRow2Cols / 4) + s * kBlk + tid];
    }
    const char* ld_row[kRows2] = {nullptr, nullptr};  // row bases of the tile being loaded, at the window's first column
    auto tile_rows = [&](int t) {
        const int2 c2 = rows_of.get2((g0 + t) * kRows2);
        const int row0 = (g0 + t) * kRows2;
        ld_row[0] = reinterpret_cast<const char*>(Yin + (size_t)c2.x * N);
        ld_row[1] = reinterpret_cast<const char*>(Yin + (size_t)(row0 + 1 < A ? c2.y : cat_last) * N);
    };
    // One 16-byte load per lane: scalar base + 32-bit lane offset.  Written as an instruction so that the
    // addresses stay out of the vector registers; the compiler therefore does not know that the result
    // arrives later, and the wait for it is written out in the main loop (wait_tile).
    auto load_piece = [&](int i) {  // piece i = row i & 1 of segment i >> 1; i is a constant wherever this is called
        const int s = i >> 1, r = i & 1;
        if (s < nseg) {
            asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(st[s][r]) : "v"(off[s]), "s"(ld_row[r]) : "memory");
        }
    };
    auto wait_tile = [&]() {  // every load (and store) issued so far has completed; the staged values may be touched
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int s = 0; s < 4; ++s) asm volatile("" : "+v"(st[s][0]), "+v"(st[s][1]));
    };
    // The eight loads of a tile are issued back to back.  The memory pipeline accepts them only as fast as
    // L2 delivers (about 22 bytes per clock and CU), so the last wave starts computing some 6000 clocks
    // after the first; spreading the loads over the compute phase instead was measured slower (every wave
    // then waits at every load).
    auto load_tile = [&](int t) {
        tile_rows(t);
        load_piece(0);
        load_piece(1);
        load_piece(2);
        load_piece(3);
        load_piece(4);
        load_piece(5);
        load_piece(6);
        load_piece(7);
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (s < nseg) {
                const uint32_t a = st_addr + (uint32_t)s * (kRow2Seg * 8u);
                *reinterpret_cast<lds_f2*>(a + 0 * 256) = f32x2{st[s][0].x, st[s][1].x};
                *reinterpret_cast<lds_f2*>(a + 1 * 256) = f32x2{st[s][0].y, st[s][1].y};
                *reinterpret_cast<lds_f2*>(a + 2 * 256) = f32x2{st[s][0].z, st[s][1].z};
                *reinterpret_cast<lds_f2*>(a + 3 * 256) = f32x2{st[s][0].w, st[s][1].w};
            }
        }
    };

    // my four biases wait in LDS behind the tile (registers are what this kernel is short of)
    using lds_f1 = __attribute__((address_space(3))) float;
    const uint32_t bias_addr = lds_base + kRow2TileBytes + 4u * tid;
#pragma unroll
    for (int s = 0; s < 4; ++s)
        *reinterpret_cast<lds_f1*>(bias_addr + s * (4 * kBlk)) = bias[unit_neuron(u, s * kBlk + tid, w.seg_log2, w.seg_stride)];
    // Output: after the transpose lane 4q+i holds row (i & 1) of the unit's neurons p .. p+3 (four neighbours: a
    // segment is a multiple of 4 long), p = (2h + (i >> 1)) * 1024 + 4q.  p for h = 0; the byte offset of the
    // 16-byte piece from the start of the row group's first output row is worked out per tile (one register here).
    const uint32_t out_p = (uint32_t)(((lane >> 1) & 1) * kBlk + (tid & ~3));
    const uint32_t out_row_off = 4u * (uint32_t)(lane & 1) * (uint32_t)N;

    load_tile(0);
    wait_tile();
    store_tile();
    __syncthreads();
    for (int t = 0; t < T; ++t) {
        const int row0 = (g0 + t) * kRows2;
        const int nlive = min(kRows2, A - row0);
        char* out_row = reinterpret_cast<char*>(Yout + (size_t)row0 * N);
        unsigned pos = 0;
        const bool more = t + 1 < T;
        if (more) tile_rows(t + 1);
#pragma unroll
        for (int h = 0; h < 2; ++h) {  // two neuron slots at a time: compute, then Eq. 1's bias, ReLU and clip
            // The loads of the next tile go out in kRow2Bursts bursts spread over the compute phase, one before
            // every (8 / kRow2Bursts)-th block of 16 connections.  A wave that issues loads is stuck until the
            // memory pipeline has taken them, which it does only as fast as L2 delivers (about 22 bytes per
            // clock and CU): all eight loads back to back leave the last wave 6000 clocks behind the first.
            float a0[kRows2] = {0.0f, 0.0f}, a1[kRows2] = {0.0f, 0.0f};
#pragma unroll
            for (int b = 0; b < 4; ++b) {  // block b of this pair of slots = block 4h + b of the step
                constexpr int every = 8 / kRow2Bursts;
                if (more && (4 * h + b) % every == 0) {
#pragma unroll
                    for (int i = 0; i < every; ++i) load_piece(4 * h + b + i);
                }
                fma_row2_block16(b < 2 ? a0 : a1, &p[2 * h + (b >> 1)][8 * (b & 1)], wuni, s3);
            }
            const float b0 = *reinterpret_cast<const lds_f1*>(bias_addr + (2 * h) * (4 * kBlk));
            const float b1 = *reinterpret_cast<const lds_f1*>(bias_addr + (2 * h + 1) * (4 * kBlk));
            float y0 = fminf(fmaxf(a0[0] + b0, 0.0f), kClip), y1 = fminf(fmaxf(a0[1] + b0, 0.0f), kClip);
            float y2 = fminf(fmaxf(a1[0] + b1, 0.0f), kClip), y3 = fminf(fmaxf(a1[1] + b1, 0.0f), kClip);
            pos |= (__builtin_amdgcn_ballot_w64(y0 > 0.0f || y2 > 0.0f) != 0ull ? 1u : 0u) |
                   (__builtin_amdgcn_ballot_w64(y1 > 0.0f || y3 > 0.0f) != 0ull ? 2u : 0u);
            transpose_quartet(y0, y1, y2, y3);
            if ((lane & 1) < nlive) {
                const uint32_t nrn = (uint32_t)unit_neuron(u, (int)out_p + h * (2 * kBlk), w.seg_log2, w.seg_stride);
                __builtin_nontemporal_store(f32x4{y0, y1, y2, y3}, reinterpret_cast<f32x4*>(out_row + (out_row_off + 4u * nrn)));  // see finish_rows
            }
        }
        if (lane < nlive && ((pos >> lane) & 1u)) flags[row0 + lane] = 1;  // lane r raises row r's flag
        __syncthreads();  // every wave is done reading tile t
        if (more) {
            wait_tile();
            store_tile();
            __syncthreads();
        }
    }
}

// a0 for the gathered footprint: per unit of 4096 neurons (unit_neuron), the groups of four columns
// (column >> 2) that any of its connections touches.  One workgroup per unit: a bitmap of the row's N / 4
// groups in LDS, a prefix count over it, and out come
//   map[u][g]   first column of the group that tile slot g holds,
//   rank[u][c4] tile slot of group c4 (meaningful for the groups that are used),
//   ngroups[u]  number of groups; the tile holds kRow2Cols / 4 of them.
// The i-th group in ascending order goes to slot gather_slot(i): inside every block of 32 slots (one round of
// the 32 bank pairs) the order is rotated by the block's number.  In a strided pattern a neuron's 32 columns
// sit at the same place of 32 different blocks; unrotated they would all lie in one bank pair, and the four
// neighbouring neurons that share a group of four columns would collide in every step whatever the order of
// their connections.  Slots that hold no group repeat the unit's last group (a harmless load).
__device__ __forceinline__ int gather_slot(int i) { return (i & ~31) | ((i + (i >> 5)) & 31); }
__global__ __launch_bounds__(kBlk) void row2_gather_kernel(const int32_t* __restrict__ idx, int N, int seg_log2,
                                                           int seg_stride, int32_t* __restrict__ map,
                                                           uint16_t* __restrict__ rank, int* __restrict__ ngroups) {
    __shared__ uint32_t bits[65536 / 4 / 32];  // one bit per group of four columns
    __shared__ uint32_t before[65536 / 4 / 32 + 1];
    __shared__ int last_col;
    const int u = blockIdx.x;
    const int tid = threadIdx.x;
    const int words = (N / 4 + 31) / 32;
    constexpr int kSlots = kRow2Cols / 4;
    for (int i = tid; i < words; i += kBlk) bits[i] = 0;
    if (tid == 0) last_col = 0;
    __syncthreads();
    for (int e = tid; e < kUnit4 * kNnz; e += kBlk) {
        const int c = idx[(size_t)unit_neuron(u, e / kNnz, seg_log2, seg_stride) * kNnz + (e % kNnz)];
        if (c >= 0 && c < N) atomicOr(&bits[c >> 7], 1u << ((c >> 2) & 31));  // bad columns were reported
    }
    __syncthreads();
    if (tid == 0) {  // N / 128 <= 512 words: a serial scan is short
        uint32_t run = 0;
        for (int i = 0; i < words; ++i) {
            before[i] = run;
            run += __popc(bits[i]);
        }
        before[words] = run;
        ngroups[u] = (int)run;
    }
    __syncthreads();
    const int total = (int)before[words];
    const int held = min(total, kSlots);  // a unit with more groups does not fit; the host looks at ngroups
    for (int c4 = tid; c4 < N / 4; c4 += kBlk) {
        const uint32_t wbits = bits[c4 >> 5];
        const int i = (int)before[c4 >> 5] + __popc(wbits & ((1u << (c4 & 31)) - 1u));
        if (((wbits >> (c4 & 31)) & 1u) && i == held - 1) last_col = 4 * c4;
    }
    __syncthreads();
    for (int k = tid; k < kSlots; k += kBlk) map[(size_t)u * kSlots + k] = last_col;
    __syncthreads();
    for (int c4 = tid; c4 < N / 4; c4 += kBlk) {
        const uint32_t wbits = bits[c4 >> 5];
        const int i = (int)before[c4 >> 5] + __popc(wbits & ((1u << (c4 & 31)) - 1u));
        const int g = gather_slot(min(i, kSlots - 1));
        rank[(size_t)u * (N / 4) + c4] = (uint16_t)g;
        if (((wbits >> (c4 & 31)) & 1u) && i < kSlots) map[(size_t)u * kSlots + g] = 4 * c4;
    }
}

// The sizes alone, for every segment length at once: workgroup (u, y) counts the groups of four columns that
// unit u (of `unit` neurons: 4096, or 2048 for the two-neurons-per-lane kernel) touches with segments of
// 1 << (log2(unit) - y) neurons; out[y * gridDim.x + u].
__global__ __launch_bounds__(kBlk) void row2_footprint_kernel(const int32_t* __restrict__ idx, int N, int* __restrict__ out,
                                                              int unit = kUnit4) {
    __shared__ uint32_t bits[65536 / 4 / 32];
    __shared__ int total;
    const int u = blockIdx.x;
    const int seg_log2 = (unit == kUnit4 ? kSegLog2Max : kSegLog2Max - 1) - (int)blockIdx.y;
    const int seg_stride = (N / unit) << seg_log2;
    const int tid = threadIdx.x;
    const int words = (N / 4 + 31) / 32;
    for (int i = tid; i < words; i += kBlk) bits[i] = 0;
    if (tid == 0) total = 0;
    __syncthreads();
    for (int e = tid; e < unit * kNnz; e += kBlk) {
        const int c = idx[(size_t)unit_neuron(u, e / kNnz, seg_log2, seg_stride) * kNnz + (e % kNnz)];
        if (c >= 0 && c < N) atomicOr(&bits[c >> 7], 1u << ((c >> 2) & 31));
    }
    __syncthreads();
    int mine = 0;
    for (int i = tid; i < words; i += kBlk) mine += __popc(bits[i]);
    if (mine) atomicAdd(&total, mine);
    __syncthreads();
    if (tid == 0) out[blockIdx.y * gridDim.x + u] = total;
}

// a0 for fused_row2_kernel: one wave per group of 32 neighbouring neurons of one neuron slot
// (the lanes a ds_read_b64 serves together).  Orders the group's connections so that in every
// step the 32 lanes read 32 different bank pairs whenever possible and writes the steps as 16-bit
// tile positions, eight per 16-byte word, lane-major.
//
// The ordering is order_group32's (spdnn_order.h), choice for choice, with the wave's first 32 lanes
// in two roles: lane l as the group's l-th neuron (its unplaced connections, its pair of the current
// step, its parent in the search) and lane q as bank pair q (the lanes that still have a connection
// there, how many connections, the lane it is matched with).  What the serial routine loops over --
// the 32 pairs for the most urgent one, the lanes a pair reaches, the pairs a lane may share -- is a
// wave reduction or a bit mask here; the breadth-first search itself stays serial, one pair per turn.
// One thread per group took 14 ms per 16384-neuron layer; this takes well under one.
constexpr int kRow2PackThreads = 64;
struct Pack32Scratch {
    uint32_t conn[32][32];  // [q][l]: connections (bit k) of lane l that fall in pair q
    uint32_t adj[32];       // lanes that still have a connection in pair q
    uint32_t remq[32];      // connections not placed yet in pair q, whole group
    uint32_t queue[36];
};
// over lanes 0..31: the two rows of 16, then one value from each
__device__ __forceinline__ int wave32_max(int v) {
    v = row16_max(v);
    return max(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16));
}
__device__ __forceinline__ int wave32_min(int v) {
    v = row16_min(v);
    return min(__builtin_amdgcn_readlane(v, 0), __builtin_amdgcn_readlane(v, 16));
}
__global__ __launch_bounds__(kRow2PackThreads) void row2_pack_kernel(const int32_t* __restrict__ idx, int N,
                                                                     const int2* __restrict__ win,
                                                                     const uint16_t* __restrict__ rank,  // NULL: contiguous windows
                                                                     int seg_log2, int seg_stride,
                                                                     uint16_t* __restrict__ codes) {
    __shared__ Pack32Scratch S;
    const int g = blockIdx.x;  // group: unit, slot, 32 lanes
    const int groups_per_unit = kUnit4 / kGroup32;
    const int u = g / groups_per_unit;
    if (u * kUnit4 >= N) return;
    const int in_unit = g - u * groups_per_unit;
    const int s = in_unit / (kBlk / kGroup32);
    const int lane0 = (in_unit - s * (kBlk / kGroup32)) * kGroup32;
    const int c_lo = rank ? 0 : row2_window(win, u, N).x;
    const int lane = threadIdx.x;
    const bool on = lane < 32;       // the upper half of the wave only keeps the reductions company
    const int l = lane & 31;
    const int32_t* mine = idx + (size_t)unit_neuron(u, s * kBlk + lane0 + l, seg_log2, seg_stride) * kNnz;
    auto pos_of = [&](int k) -> uint32_t {  // out-of-range columns were reported; keep them harmless
        int c = mine[k];
        if (c < 0 || c >= N) c = c_lo;
        // tile column: inside the window, or in the gathered list group rank[c >> 2], column c & 3 of it
        const uint32_t tc = rank ? 4u * rank[(size_t)u * (N / 4) + (c >> 2)] + (uint32_t)(c & 3) : (uint32_t)win_rel(c, c_lo, N);
        return row2_pos(tc & (kRow2Cols - 1));
    };
    for (int q = 0; q < 32; ++q)
        if (on) S.conn[q][l] = 0;
    if (on) {
        S.adj[l] = 0;
        S.remq[l] = 0;
    }
    __syncthreads();
    if (on)
        for (int k = 0; k < 32; ++k) {
            const int q = (int)(pos_of(k) & 31u);
            S.conn[q][l] |= 1u << k;  // my own column of the table
        }
    __syncthreads();
    if (on)
        for (int q = 0; q < 32; ++q) {
            const uint32_t m = S.conn[q][l];
            if (m) {
                atomicOr(&S.adj[q], 1u << l);
                atomicAdd(&S.remq[q], (uint32_t)__popc(m));
            }
        }
    __syncthreads();
    uint32_t unplaced = 0xFFFFFFFFu;  // lane l's connections not placed yet
    for (int step = 0; step < 32; ++step) {
        const int left = 32 - step;
        const uint32_t adj = on ? S.adj[l] : 0u;  // as pair q = l
        const int remq = on ? (int)S.remq[l] : 0;
        int lane_of_pair = -1;  // as pair
        int pair_of_lane = -1;  // as lane
        int parent = -1;        // as lane: the pair from which the search reached me
        uint32_t free_lanes = 0xFFFFFFFFu;  // lanes without a pair (the same in every lane)
        uint32_t done = 0;                  // pairs already offered
        for (int r = 0; r < 32; ++r) {
            // the most urgent pair not offered yet, the lowest-numbered one among equals
            const int key = (!on || ((done >> l) & 1u)) ? -1 : ((((remq >= left) ? 4096 : 0) + remq) << 5) | (31 - l);
            const int best = wave32_max(key);
            const int q0 = 31 - (best & 31);
            done |= 1u << q0;
            if (((best >> 5) & 4095) == 0) break;  // the rest are empty too
            // breadth-first search for an augmenting path from pair q0 to a lane without a pair
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
                        S.queue[tail + __popc(cand & ((1u << l) - 1u))] = (uint32_t)pair_of_lane;  // a lane is seen once: at most 32 entries follow q0
                    }
                    tail += __popc(cand);
                    __syncthreads();
                }
            }
            if (found < 0) continue;
            free_lanes &= ~(1u << found);
            for (int cur = found;;) {
                const int q = __builtin_amdgcn_readlane(parent, cur);
                const int next = __builtin_amdgcn_readlane(lane_of_pair, q);  // the lane that gives q up (meaningful unless q == q0)
                if (lane == q) lane_of_pair = cur;
                if (lane == cur) pair_of_lane = q;
                if (q == q0) break;
                cur = next;
            }
        }
        // a lane left without a pair of its own shares the least used pair it can, lanes in ascending order
        int mult = (on && lane_of_pair >= 0) ? 1 : 0;  // as pair: lanes using me in this step
        for (uint32_t rest = free_lanes; rest;) {
            const int ll = __builtin_ctz(rest);
            rest &= rest - 1;
            const int key = (on && ((adj >> ll) & 1u)) ? ((mult * 65536 - remq + 2048) << 5) | l : 0x7fffffff;
            const int bq = wave32_min(key) & 31;
            if (lane == ll) pair_of_lane = bq;
            if (lane == bq) ++mult;
        }
        // place: the lowest unplaced connection of my pair
        if (on) {
            const uint32_t in_pair = S.conn[pair_of_lane][l];
            const int k = __builtin_ctz(in_pair & unplaced);
            unplaced &= ~(1u << k);
            atomicSub(&S.remq[pair_of_lane], 1u);
            if ((in_pair & unplaced) == 0) atomicAnd(&S.adj[pair_of_lane], ~(1u << l));
            const size_t word = ((size_t)(u * 4 + s) * 4 + (step >> 3)) * kBlk + lane0 + l;
            codes[word * 8 + (step & 7)] = (uint16_t)pos_of(k);
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// a0: new names for neurons and columns, so that a strided layer fits the two-neurons-per-lane kernel
// (PairRelabel).  Units of kPairUnit neurons in segments (unit_neuron); if the units' columns do not overlap and
// no unit reads more than kPairUnit columns, unit u's groups of four columns get the new names u * kPairUnit / 4 + rank
// (ascending), its neurons the new numbers u * kPairUnit + local index, and under the new names every unit has a
// contiguous window of at most kPairUnit columns: an ordinary layer for the set-up and the kernel.
// ---------------------------------------------------------------------------
constexpr int kPairUnit = 2 * kBlk;

// owner[g] = the unit that reads group g (-1: none); *conflict = 1 if two units read the same group.
__global__ __launch_bounds__(kBlk) void relabel_owner_kernel(const int32_t* __restrict__ idx, int N, int seg_log2,
                                                             int seg_stride, int* __restrict__ owner,
                                                             int* __restrict__ conflict) {
    const int u = blockIdx.x;
    for (int e = threadIdx.x; e < kPairUnit * kNnz; e += kBlk) {
        const int c = idx[(size_t)unit_neuron(u, e / kNnz, seg_log2, seg_stride) * kNnz + (e % kNnz)];
        if (c < 0 || c >= N) continue;  // reported by the window scan
        const int old = atomicCAS(&owner[c >> 2], -1, u);
        if (old != -1 && old != u) *conflict = 1;
    }
}

// Unit u's groups in ascending order: newname[g] = u * (kPairUnit / 4) + rank, col[that] = 4 g; names of the unit
// that no group got point at the unit's last group (or column 0).  *conflict = 1 if a unit has more than
// kPairUnit / 4 groups.
__global__ __launch_bounds__(kBlk) void relabel_rank_kernel(const int* __restrict__ owner, int N, int* __restrict__ newname,
                                                            int32_t* __restrict__ col, int* __restrict__ conflict) {
    __shared__ int wave_cnt[17];
    __shared__ int s_max;
    const int u = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    constexpr int cap = kPairUnit / 4;
    int base = 0;
    for (int g0 = 0; g0 < N / 4; g0 += kBlk) {
        const int g = g0 + tid;
        const bool mine = g < N / 4 && owner[g] == u;
        const unsigned long long m = __builtin_amdgcn_ballot_w64(mine);
        __syncthreads();
        if (lane == 0) wave_cnt[wave] = __popcll(m);
        __syncthreads();
        if (tid == 0) {
            int run = 0;
            for (int k = 0; k < 16; ++k) {
                const int v = wave_cnt[k];
                wave_cnt[k] = run;
                run += v;
            }
            wave_cnt[16] = run;
        }
        __syncthreads();
        if (mine) {
            const int r = base + wave_cnt[wave] + __popcll(m & ((1ull << lane) - 1ull));
            if (r < cap) {
                newname[g] = u * cap + r;
                col[u * cap + r] = 4 * g;
            } else {
                *conflict = 1;
            }
        }
        base += wave_cnt[16];
    }
    __syncthreads();
    // the names past the unit's last group: any of its columns will do (a harmless load); take its largest
    if (base < cap) {
        if (tid == 0) s_max = 0;
        __syncthreads();
        for (int r = tid; r < base; r += kBlk) atomicMax(&s_max, col[u * cap + r]);
        __syncthreads();
        for (int r = base + tid; r < cap; r += kBlk) col[u * cap + r] = s_max;
    }
}

// The layer under the new names: row u * kPairUnit + p = the connections of unit u's p-th neuron, every column
// by its new name (columns out of range are passed through, for the window scan to report).
__global__ void relabel_apply_kernel(const int32_t* __restrict__ idx, int N, int seg_log2, int seg_stride,
                                     const int* __restrict__ newname, int32_t* __restrict__ out_idx) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)N * kNnz) return;
    const int v = (int)(i / kNnz), k = (int)(i % kNnz);
    const int c = idx[(size_t)unit_neuron(v / kPairUnit, v % kPairUnit, seg_log2, seg_stride) * kNnz + k];
    out_idx[i] = (c >= 0 && c < N) ? 4 * newname[c >> 2] + (c & 3) : c;
}

}  // namespace spdnn
