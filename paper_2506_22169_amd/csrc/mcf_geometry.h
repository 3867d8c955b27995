// Tile geometry shared by the kernels and the host-side budget checks: LDS row pitches and
// sizes.  Plain constexpr C++, no HIP.
#pragma once

namespace mcf {

// Row pitch in bytes of an LDS tile that is read with the transposing 64-bit LDS read
// (rows of `elems` 16-bit elements).  Half a wave reads 4 rows x 64 B at once; an odd
// multiple of 64 B puts those four pieces on disjoint banks.
constexpr int pitch_tr(int elems) {
    int p = elems * 2;
    return (p % 128 == 64) ? p : (p / 128) * 128 + 64 + ((p % 128 > 64) ? 128 : 0);
}

// Row pitch in bytes of the K-contiguous B tile (read with plain 128-bit LDS reads).
constexpr int pitch_bk(int K) { return K * 2 + 16; }

constexpr int b_tile_bytes(int K, int tn, bool b_kcontig) {
    return b_kcontig ? tn * pitch_bk(K) : K * pitch_tr(tn);
}
constexpr int d_tile_bytes(int L, int tn) { return tn * pitch_tr(L); }
constexpr int stage_bytes(int K, int L, int tn, bool b_kcontig) {
    return b_tile_bytes(K, tn, b_kcontig) + d_tile_bytes(L, tn);
}
// Scratch for the cross-wave combine when ns > 1: per row-group, (ns-1) waves park their E
// accumulators (fp32) and softmax state.
constexpr int combine_bytes(int L, int mb, int rg, int ns) {
    return ns > 1 ? rg * (ns - 1) * mb * ((L / 32) * 16 + 2) * 64 * 4 : 0;
}
constexpr int total_lds_bytes(int K, int L, int mb, int rg, int ns, bool b_kcontig) {
    int s = 2 * stage_bytes(K, L, 32 * ns, b_kcontig);
    int c = combine_bytes(L, mb, rg, ns);
    return s > c ? s : c;
}

} // namespace mcf
