// Packed sign bits -> FP4 operands of the matrix-core convolution, and the layout of the expanded
// filter workspace.  Shared by the convolution (which expands input words while staging them) and
// by the two kernels that can fill the filter workspace.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace xnor {

// Four bit pairs (one per byte of `sel`, values 0..3) -> four bytes of two FP4 codes each
// (bit 1 -> 0x2 = +1.0, bit 0 -> 0xA = -1.0; the pair's low bit is the low nibble): a four-entry
// byte table looked up through v_perm_b32.
__device__ inline uint32_t pair_codes(uint32_t sel)
{
    return __builtin_amdgcn_perm(0u, 0x222AA2AAu, sel);
}

// One packed word -> 32 FP4 values in four registers; `nvalid` channels are real, the rest become
// FP4 zero.  Register j, byte k holds channels 8k+2j (low nibble) and 8k+2j+1 (high nibble) of the
// word, which costs a shift, a mask and a lookup per register.  The order of the 32 values inside
// a register quad is free: both MFMA operands are expanded by this one function, so value i of a
// pixel always meets value i of a filter, and the sum of the products does not depend on i's order.
__device__ inline uint4 expand_word(uint32_t w, int nvalid)
{
    uint4 e;
    e.x = pair_codes(w & 0x03030303u);
    e.y = pair_codes((w >> 2) & 0x03030303u);
    e.z = pair_codes((w >> 4) & 0x03030303u);
    e.w = pair_codes((w >> 6) & 0x03030303u);
    if (nvalid < 32) {
        auto m = [&](int j) -> uint32_t {
            uint32_t keep = 0;
            for (int k = 0; k < 4; ++k) {
                if (8 * k + 2 * j < nvalid) keep |= 0x0fu << (8 * k);
                if (8 * k + 2 * j + 1 < nvalid) keep |= 0xf0u << (8 * k);
            }
            return keep;
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
