// Tile geometry shared by the kernels and the host-side budget checks: tile byte sizes, the
// XOR swizzles of the LDS layouts and the LDS total.  Plain constexpr C++, no HIP.
#pragma once

namespace mcf {

// All LDS tiles keep their natural row pitch (row bytes RB, a power of two >= 64) and are
// filled by direct global->LDS loads in units of 16-byte chunks; bank conflicts are avoided
// by XOR-ing the chunk index within a row with a function of the row.
//
// Tiles read with plain 128-bit reads (A tile; B tile when K is contiguous): 16 consecutive
// rows are read at the same logical chunk, so consecutive rows must land on distinct 16-byte
// bank groups of the 256-byte LDS line.
constexpr int swz_b128(int row_bytes, int row) {
    return row_bytes == 64 ? ((row >> 2) & 3) : row_bytes == 128 ? ((row >> 1) & 7) : (row & 15);
}
// Tiles read with the transposing 64-bit read (D tile; B tile when N is contiguous): half a
// wave reads 4 consecutive rows x 64 bytes, so the four rows must land on distinct 64-byte
// groups.  Returned as a chunk mask (multiple of 4 chunks = 64 bytes).
constexpr int swz_tr(int row_bytes, int row) {
    return row_bytes == 64 ? 0 : row_bytes == 128 ? 4 * ((row >> 1) & 1) : 4 * (row & 3);
}

// K and L need not be powers of two (K a multiple of 16, L of 8): rows of the LDS tiles are
// then laid out with the next power-of-two pitch (the swizzles want one); the chunks beyond
// K or L in a row are loaded from valid memory and never reach a result that is stored.
constexpr int pitch_elems(int x) { return x <= 32 ? 32 : x <= 64 ? 64 : x <= 128 ? 128 : x <= 256 ? 256 : 512; }
constexpr int h_blocks(int L) { return (L + 31) / 32; } // 32-wide column blocks of E (the last may be partial)

constexpr int a_tile_bytes(int K, int mb, int rg) { return 32 * mb * rg * pitch_elems(K) * 2; }
constexpr int b_tile_bytes(int K, int tn) { return pitch_elems(K) * tn * 2; }
constexpr int d_tile_bytes(int L, int tn) { return tn * pitch_elems(L) * 2; }
constexpr int stage_bytes(int K, int L, int tn) { return b_tile_bytes(K, tn) + d_tile_bytes(L, tn); }
// Cross-wave combine when ns > 1: the mb * ceil(L/32) accumulator blocks (32 x 32 of E, 16 fp32
// per lane) of a row-group are dealt out to its ns waves, BPW in a row; every wave parks the
// blocks it does not own and its softmax state in LDS.
constexpr int blocks_per_wave(int L, int mb, int ns) { return (mb * h_blocks(L) + ns - 1) / ns; }
// Most blocks any wave parks: all but the run it owns; the last wave's run is the shortest
// (empty when there are fewer blocks than waves).
constexpr int parked_blocks(int L, int mb, int ns) {
    const int n = mb * h_blocks(L), bpw = blocks_per_wave(L, mb, ns);
    const int last = n - (ns - 1) * bpw;
    return n - (last < 0 ? 0 : last);
}
// A wave's run of blocks must lie within one row set of 32 rows or cover whole row sets.
constexpr bool combine_runs_ok(int L, int mb, int ns) {
    const int hb = h_blocks(L), bpw = blocks_per_wave(L, mb, ns);
    return bpw >= hb ? bpw % hb == 0 : (mb == 1 || hb % bpw == 0);
}
constexpr int combine_bytes(int L, int mb, int rg, int ns) {
    return ns > 1 ? rg * ns * (parked_blocks(L, mb, ns) * 16 + 2 * mb) * 64 * 4 : 0;
}
// Staging tile of the E store, per wave: the rows of the row sets it owns (32 each) times the
// bytes of the h blocks it owns in a row, that pitch rounded up to a power of two.
constexpr int estage_row_bytes(int L, int mb, int ns) {
    const int hb = h_blocks(L), bpw = blocks_per_wave(L, mb, ns);
    const int hpw = bpw < hb ? bpw : hb;
    return 2 * pitch_elems(32 * hpw);
}
constexpr int estage_wave_bytes(int L, int mb, int ns) {
    const int hb = h_blocks(L), bpw = blocks_per_wave(L, mb, ns);
    const int mpw = bpw < hb ? 1 : bpw / hb;
    return mpw * 32 * estage_row_bytes(L, mb, ns);
}
constexpr int estage_bytes(int L, int mb, int rg, int ns) { return rg * ns * estage_wave_bytes(L, mb, ns); }
// Kernels with a k loop inside the block (T_K < K; `K` below is then the chunk T_K): the ring
// carries two kinds of items, an A chunk + B chunk (tm x T_K, T_K x tn) per k step and the D
// tile once per n-tile; a slot is as large as the larger of the two.
constexpr int ksplit_slot_bytes(int TK, int L, int mb, int rg, int tn) {
    const int ab = a_tile_bytes(TK, mb, rg) + b_tile_bytes(TK, tn), d = d_tile_bytes(L, tn);
    return ab > d ? ab : d;
}
// `stages` ring buffers of one B + D tile each; the A tile is staged in the last ring slot
// (it is consumed before that slot is first filled); after the loop the ring space is reused
// by the combine scratch followed by the staging tiles of the E store.
constexpr int total_lds_bytes(int K, int L, int mb, int rg, int ns, int nj, int stages, bool ksplit = false) {
    const int st = stage_bytes(K, L, 32 * ns * nj);
    const int a = a_tile_bytes(K, mb, rg);
    int s = ksplit ? stages * ksplit_slot_bytes(K, L, mb, rg, 32 * ns * nj) : (stages - 1) * st + (a > st ? a : st);
    const int c = combine_bytes(L, mb, rg, ns) + estage_bytes(L, mb, rg, ns);
    return s > c ? s : c;
}
// Three-GEMM chain (E . F with F[L x P] after the loop): the F tile sits behind everything else
// for the whole life of the block; the output tile is combined and staged like E.
constexpr int chain3_f_bytes(int L, int P) { return L * pitch_elems(P) * 2; }
constexpr int chain3_f_offset(int K, int L, int P, int mb, int rg, int ns, int nj, int stages) {
    const int t = total_lds_bytes(K, L, mb, rg, ns, nj, stages);
    const int e = combine_bytes(P, mb, rg, ns) + estage_bytes(P, mb, rg, ns);
    return ((t > e ? t : e) + 1023) / 1024 * 1024;
}
constexpr int chain3_lds_bytes(int K, int L, int P, int mb, int rg, int ns, int nj, int stages) {
    return chain3_f_offset(K, L, P, mb, rg, ns, nj, stages) + chain3_f_bytes(L, P);
}
// Largest ring depth (2..4) that keeps a block within `budget` bytes of LDS.
constexpr int pick_stages(int K, int L, int mb, int rg, int ns, int nj, int budget, bool ksplit = false) {
    int s = 4;
    while (s > 2 && total_lds_bytes(K, L, mb, rg, ns, nj, s, ksplit) > budget) --s;
    return s;
}

// Ring depth every kernel variant is built with: as deep (up to 4) as fits 80 KiB, so that two
// blocks can share the 160 KiB LDS of a compute unit (measured: a deeper ring that costs the
// second resident block loses more than it gains).
constexpr int kLdsRingBudget = 80 * 1024;
// Softmax chains (and the plain chains named below) run a software pipeline over three consecutive n-tiles: in iteration i a wave
// issues the MFMAs of GEMM 2 of tile i-1 and of GEMM 1 of tile i+1 with the softmax arithmetic of
// tile i spread between them, so tiles i-1, i and i+1 are live and tile i+2 is landing: a ring of
// 4 (measured: a deeper one is slower, by up to a fifth on the short attention shapes).
// 0 = the arrangement cannot be pipelined because four stages do not fit the compute unit (its
// softmax loop then runs the phases one after the other, see skewed_groups).  `extra` = LDS held
// beside the ring (the F tile of a three-GEMM chain).
constexpr int pipe_stages(int K, int L, int mb, int rg, int ns, int nj, bool softmax, bool ksplit = false, int extra = 0) {
    if (ksplit) return 0;
    // plain chains: only where K and L are 32, in blocks of 8 waves that own at most two row sets
    // each (measured on 16 x [4096,32].[32,1024].[1024,32]: 3-4 % faster for (1,8,1,2) and (2,4,2,2),
    // no change for (1,4,2,2), a third slower for (4,2,4,1); with K = L = 64 slower throughout)
    if (!softmax && !(K <= 32 && L <= 32 && mb <= 2 && rg * ns == 8)) return 0;
    return total_lds_bytes(K, L, mb, rg, ns, nj, 4) + extra <= 160 * 1024 ? 4 : 0;
}
// Waves per SIMD a pipelined softmax kernel is compiled for.  A block brings rg*ns/4 of them; a
// second resident block hides the block's barriers and the ends of its pipeline (measured: a
// third to a half faster on the short attention shapes), but the compiler only keeps to the
// registers that leaves a wave (512 / waves) when told so, otherwise it drifts a few registers
// over.  Asked for when two blocks fit the LDS and the tiles a lane must hold (the E
// accumulators, two C^T tiles, P packed to 16 bit) leave some 56 registers for operands,
// addresses and the softmax state.
constexpr int pipe_waves_per_simd(int K, int L, int mb, int rg, int ns, int nj, int extra = 0) {
    const int per_block = rg * ns >= 4 ? rg * ns / 4 : 1;
    if (2 * (total_lds_bytes(K, L, mb, rg, ns, nj, 4) + extra) > 160 * 1024) return per_block;
    const int held = mb * h_blocks(L) * 16 + 2 * nj * mb * 16 + nj * mb * 8;
    return held + 56 <= 512 / (2 * per_block) ? 2 * per_block : per_block;
}
// Softmax chains that cannot be pipelined, in blocks of 8 waves, run their two wave groups a
// phase apart, which keeps two n-tiles live: their ring is at least 3 deep.
constexpr bool skewed_groups(int rg, int ns, bool softmax, bool ksplit = false) { return softmax && rg * ns == 8 && !ksplit; }
constexpr int ring_stages(int K, int L, int mb, int rg, int ns, int nj, bool softmax, bool ksplit = false, int extra = 0) {
    // the items of a k loop are small and many, and the shapes that need one rarely fill the
    // machine: as deep as the whole LDS allows, to keep as many loads in flight as possible
    if (ksplit) return pick_stages(K, L, mb, rg, ns, nj, 2 * kLdsRingBudget, true);
    const int ps = pipe_stages(K, L, mb, rg, ns, nj, softmax, ksplit, extra);
    if (ps) return ps;
    const int s = pick_stages(K, L, mb, rg, ns, nj, kLdsRingBudget);
    return (skewed_groups(rg, ns, softmax) && s < 3) ? 3 : s;
}

} // namespace mcf
