// Packed sign bits -> FP4 operands of the matrix-core convolution, and the layout of the expanded
// filter workspace.  Shared by the convolution (which expands input words while staging them) and
// by the two kernels that can fill the filter workspace.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace xnor {

// 8 sign bits -> 8 FP4 codes (bit 1 -> 0x2 = +1.0, bit 0 -> 0xA = -1.0); channel i -> nibble i.
// Two bits select one byte of a four-entry table through v_perm_b32.
__device__ inline uint32_t expand8(uint32_t b)
{
    uint32_t t = b | (b << 6);
    t |= t << 12;
    t &= 0x03030303u;
    return __builtin_amdgcn_perm(0u, 0x222AA2AAu, t);
}

// One packed word -> 32 FP4 values; `nvalid` channels are real, the rest become FP4 zero.
__device__ inline uint4 expand_word(uint32_t w, int nvalid)
{
    uint4 e;
    e.x = expand8(w & 0xffu);
    e.y = expand8((w >> 8) & 0xffu);
    e.z = expand8((w >> 16) & 0xffu);
    e.w = expand8(w >> 24);
    if (nvalid < 32) {
        auto m = [&](int d) -> uint32_t {
            const int nv = nvalid - 8 * d;
            return nv >= 8 ? 0xffffffffu : (nv <= 0 ? 0u : ((1u << (4 * nv)) - 1u));
        };
        e.x &= m(0); e.y &= m(1); e.z &= m(2); e.w &= m(3);
    }
    return e;
}

// Filter workspace Wx[tile32][step][lane] (one uint4 per lane): the steps of a tile run
// chunk-major, then tap-major, each chunk padded with zero steps to a whole number of register
// rings: step = chunk*chunk_pad + tap*steps_c + s, packed word = chunk*CH + 2*s + lane/32,
// filter = 32*tile32 + lane%32.  Padding steps, filters >= F, words >= Cw and channels >= C are zeros.
struct ExpandLayout {
    int ok;            // 0: the matrix-core kernel does not take the shape
    int CH, nchunks, chunk_pad, tile_steps, Cw2;
    size_t ws_bytes;
};

// The value of entry (step, kg) of filter row `f`'s lanes: `word_of(tap, w)` returns the filter's
// packed word.
template <class WordOf>
__device__ inline uint4 expanded_entry(const ExpandLayout &L, int step, int kg, int taps, int Cw, int C,
                                       WordOf word_of)
{
    uint4 v = make_uint4(0, 0, 0, 0);
    const int chunk = step / L.chunk_pad;
    if (chunk < L.nchunks) {
        const int rem = step - chunk * L.chunk_pad;
        const int steps_c = min(L.CH, L.Cw2 - chunk * L.CH) >> 1;
        if (rem < taps * steps_c) {
            const int tap = rem / steps_c, s = rem - tap * steps_c;
            const int w = chunk * L.CH + 2 * s + kg;
            if (w < Cw) v = expand_word(word_of(tap, w), min(32, C - 32 * w));
        }
    }
    return v;
}

}  // namespace xnor
