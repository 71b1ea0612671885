// Host run of the bitsliced AES-128 (dash_aes_sliced.h): 32 blocks at a time, under the sanitizers.
// Test code, not part of libdash.
//
// usage: aes_sliced_emul <in.bin> <out.bin>     in: u8 key[16]; u8 blocks[n][16], n a multiple of 32;  out: u8 blocks[n][16]
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <vector>

#include "../paper_2302_06361_amd/csrc/dash_aes_sliced.h"
#include "../paper_2302_06361_amd/csrc/dash_hostconst.h"

using namespace dash;
using namespace dash::hostconst;

int main(int argc, char** argv) {
    if (argc != 3) return 2;
    FILE* f = fopen(argv[1], "rb");
    if (!f) return 2;
    uint8_t key[16];
    if (fread(key, 1, 16, f) != 16) return 2;
    std::vector<uint8_t> in;
    uint8_t buf[512];
    size_t got;
    while ((got = fread(buf, 1, sizeof(buf), f)) > 0) in.insert(in.end(), buf, buf + got);
    fclose(f);
    if (in.size() % 512) return 2;
    uint8_t S[256];
    make_sbox(S);
    uint32_t rk[44];
    expand_key(key, S, rk);
    std::vector<uint32_t> km(9 * 128);
    sliced_key_masks(rk, km.data());

    // the transposition is what it says
    {
        uint32_t a[32], b[32];
        for (int j = 0; j < 32; j++) a[j] = b[j] = 0x9e3779b9u * (uint32_t)(j + 1) ^ (0x85ebca6bu >> (j % 13));
        transpose32(b);
        for (int t = 0; t < 32; t++)
            for (int j = 0; j < 32; j++)
                if (((b[t] >> j) & 1u) != ((a[j] >> t) & 1u)) { fprintf(stderr, "transpose32 wrong at %d %d\n", t, j); return 3; }
    }

    std::vector<uint8_t> out(in.size());
    for (size_t g = 0; g < in.size() / 512; g++) {
        uint32_t X[128];
        for (int j = 0; j < 32; j++)
            for (int w = 0; w < 4; w++) memcpy(&X[32 * w + j], &in[g * 512 + j * 16 + 4 * w], 4);
        aes128_encrypt_sliced(X, rk, km.data());
        for (int j = 0; j < 32; j++)
            for (int w = 0; w < 4; w++) memcpy(&out[g * 512 + j * 16 + 4 * w], &X[32 * w + j], 4);
    }
    f = fopen(argv[2], "wb");
    if (!f) return 2;
    fwrite(out.data(), 1, out.size(), f);
    fclose(f);
    return 0;
}
