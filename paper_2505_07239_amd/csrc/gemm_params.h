// Operand description shared by the two implementations of a party's output share
// (the matrix-core kernel for tall activations and the vector-ALU kernel for a few rows).
#pragma once

#include "common.h"

constexpr int KIND_SOMM = 0;
constexpr int KIND_SIMM = 1;

struct GemmParams {
    int kind, party;
    int m;          // rows of X / Z
    int kc_cap;     // contraction length bound: SOMM k, SIMM n_blk_cap * bs
    int n_cap;      // output width bound: SOMM n_blk_cap * bs, SIMM n
    int bs, n_blk_cap;
    int bs_shift;   // log2(bs) when bs is a power of two, else -1
    int full_extent; // length of the axis blk_idx refers to (neurons)
    const int* blk_idx;
    const int* n_blk_dev;
    // X side
    const u64* E;  long lde;
    const u64* A;  long lda;  int a_full;
    // W side
    const u64* B;  long ldb;  int b_full;
    const u64* F;  long ldf;
    const u64* F2;  // few-row path only: second masked share of the weights, F = F + F2 formed on the fly (else null)
    int w_tr;       // SOMM: B_i and F are stored neuron-major (one row of k words per output column)
    int w_planes;   // B_i and F are digit planes (comet_open_weight_planes); ldb / ldf = their columns
    const u64* C;
    u64* Z;        long ldz;
    // packed digit planes of [E | A']
    unsigned char* xp;
    int mpad;       // rows of xp, multiple of 128
    int chunk;      // contraction steps per scheduling slice, 1 .. MAX_SEG
    int ks_cap;     // contraction steps per half, ceil(kc_cap / 32)
    // general forms of Protocols 2 and 3 (null when unused)
    const int* row_comp;      // SOMM blocks: component number of each listed row
    const int* blk_comp;      // SOMM blocks: component number of each listed block
    const int* n_row_dev;     // SOMM blocks: number of listed rows (device), or null
    int* tile_list;           // SOMM blocks: output tiles that touch a result block, [0] = their count
    const int* tile_sel;      // SOMM blocks: which of two tile shapes runs (device), or null
    int tile_sel_want;        //              the value this launch answers to
    const unsigned char* tmask;   // SIMM masked: m x tmask_nb bytes, token r uses block b
    // SIMM masked, matrix-core kernel: per row tile the contraction steps that some token of
    // the tile takes part in.  step_cnt[tm] steps, listed ascending at step_list[tm * ks_cap ..];
    // step_off[tm] = number of listed steps of the row tiles before tm.
    int* step_cnt;
    int* step_off;
    int* step_list;
    long tmask_nb;
    // launch shape of the matrix-core kernel, fixed on the host before the packing kernel runs
    int grid;                 // workgroups
    int tile_bm, tile_bn;     // output tile
    int own_try;              // plain product (no result blocks, no step lists, default slicing)
    int k_rotate;             // units tile by tile; the parts of a tile take its steps in reverse order (see gemm_sweep)
    int team;                 // group launch: workgroups form teams over the row tiles (see ring_gemm_group_kernel)
    int group_n;              // members of the group launch this product is part of (0 or 1: on its own)
};

static __device__ __forceinline__ int n_blocks(const GemmParams& p) {
    int nb = p.n_blk_cap;
    if (p.n_blk_dev) {
        const int d = *p.n_blk_dev;
        nb = d < 0 ? 0 : (d < nb ? d : nb);
    }
    return nb;
}

// rows that take part: all m, or the device-resident count of listed rows
static __device__ __forceinline__ int n_rows(const GemmParams& p) {
    int m = p.m;
    if (p.n_row_dev) {
        const int d = *p.n_row_dev;
        m = d < 0 ? 0 : (d < m ? d : m);
    }
    return m;
}

// does token `row` use listed block `blk`?  (SIMM with per-token row sets)
static __device__ __forceinline__ bool token_uses(const GemmParams& p, int row, int blk) {
    const long b = p.blk_idx[blk];
    return b >= 0 && b < p.tmask_nb && p.tmask[(long)row * p.tmask_nb + b] != 0;
}

// Does every workgroup of the matrix-core kernel get whole output tiles (all of their contraction)?
// Then a tile has one writer: the kernel stores Z = C + sum directly and the packing kernel leaves Z
// alone; otherwise Z starts out as C and the slices of a tile meet in it through atomic adds.
// Both kernels evaluate this with the same device-resident counts.
static __device__ __forceinline__ bool owns_tiles(const GemmParams& p, int m_eff, int n_eff, int kc) {
    if (!p.own_try || kc <= 0 || m_eff <= 0 || n_eff <= 0) return false;
    const long tiles = (long)((m_eff + p.tile_bm - 1) / p.tile_bm) * ((n_eff + p.tile_bn - 1) / p.tile_bn);
    // (the members of a group have one shape and follow each other tile by tile)
    return tiles * (p.group_n > 1 ? p.group_n : 1) % p.grid == 0;
}

// Start of block `blk` on the indexed axis, or -1 when the id does not fit the
// axis.  Callers clamp such a block to the start of the axis: a bad id can make
// the outputs it feeds meaningless, but it can never make an access fault.
static __device__ __forceinline__ long block_start(const GemmParams& p, int blk) {
    const long s = (long)p.blk_idx[blk] * p.bs;
    return (s < 0 || s + p.bs > p.full_extent) ? -1 : s;
}

// Vector-ALU path for at most COMET_SKINNY_MAX_ROWS activation rows (decoding): computes the
// whole share, Z := C included.  p.xp is the workspace of the matrix-core path, which is
// always large enough.  Up to 8 rows it reads the weights at the rate of a device copy; from 9
// rows on its multiply-adds (three per row and weight word) take longer than the memory
// traffic and the matrix-core kernel's 32-row tile is faster.
static const int COMET_SKINNY_MAX_ROWS = 8;
int comet_launch_skinny(comet_ctx* ctx, const char* what, const GemmParams& p);

// Matrix-core path for at most COMET_FEWROW_MAX_ROWS activation rows with the weight side in digit
// planes (plain products only: no result blocks, no per-token row sets): every wavefront streams
// its own weight fragments from memory into registers.  Runs after the packing kernel (digit
// planes of [E | A'] in p.xp, Z := C).
static const int COMET_FEWROW_MAX_ROWS = 32;
int comet_launch_fewrow(comet_ctx* ctx, const char* what, const GemmParams& p);
