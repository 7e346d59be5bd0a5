// Host build of the bit-plane AES engine (csrc/aes_bitplane.h) for CPU-side unit tests.
#include <stdint.h>
#include <string.h>

#include "../paper_2006_04593_amd/csrc/aes_bitplane.h"

using namespace fss::bp;

extern "C" {

// out[j] = E_k(in[j]) ^ in[j] for eight 16-byte blocks; mode as in fss::bp::KeyMode
int bp_mmo8(int mode, const uint8_t *in, uint32_t pick, uint8_t *out)
{
    W a[8][4], o[8][4];
    memcpy(a, in, 128);
    switch (mode) {
    case 0: mmo8<kUniform0>(o, a, pick); break;
    case 1: mmo8<kUniform1>(o, a, pick); break;
    case 2: mmo8<kUniform2>(o, a, pick); break;
    case 3: mmo8<kPickLowK3High>(o, a, pick); break;
    case 4: mmo8<kPickAll>(o, a, pick); break;
    default: return -1;
    }
    memcpy(out, o, 128);
    return 0;
}

// pack then unpack must be the identity
void bp_roundtrip(const uint8_t *in, uint8_t *out)
{
    W a[8][4], o[8][4];
    memcpy(a, in, 128);
    Planes s;
    pack(s, a);
    unpack(o, s);
    memcpy(out, o, 128);
}

// S-box of every byte of eight blocks, through the circuit
void bp_subbytes(const uint8_t *in, uint8_t *out)
{
    W a[8][4], o[8][4];
    memcpy(a, in, 128);
    Planes s;
    pack(s, a);
    sub_bytes(s);
    unpack(o, s);
    memcpy(out, o, 128);
}

uint8_t bp_table_sbox(int v) { return fss::kAes.sbox[v & 255]; }

}  // extern "C"
