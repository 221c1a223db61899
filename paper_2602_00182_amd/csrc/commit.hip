// Output commitment on the host: SHA-256 as in FIPS 180-4, and the digest the paper records per
// execution, SHA256(prompt || logits || tokens) (section 6.7), over caller-provided host bytes.
// Host code only: hashing is a serial chain of 64-byte blocks, which one CPU core with the SHA
// extensions does at GB/s and a GPU thread at MB/s.
#include <immintrin.h>
#include <stdint.h>
#include <string.h>

#include "../../include/detinfer.h"

namespace {

const uint32_t kK[64] = {
    0x428a2f98, 0x71374491, 0xb5c0fbcf, 0xe9b5dba5, 0x3956c25b, 0x59f111f1, 0x923f82a4, 0xab1c5ed5,
    0xd807aa98, 0x12835b01, 0x243185be, 0x550c7dc3, 0x72be5d74, 0x80deb1fe, 0x9bdc06a7, 0xc19bf174,
    0xe49b69c1, 0xefbe4786, 0x0fc19dc6, 0x240ca1cc, 0x2de92c6f, 0x4a7484aa, 0x5cb0a9dc, 0x76f988da,
    0x983e5152, 0xa831c66d, 0xb00327c8, 0xbf597fc7, 0xc6e00bf3, 0xd5a79147, 0x06ca6351, 0x14292967,
    0x27b70a85, 0x2e1b2138, 0x4d2c6dfc, 0x53380d13, 0x650a7354, 0x766a0abb, 0x81c2c92e, 0x92722c85,
    0xa2bfe8a1, 0xa81a664b, 0xc24b8b70, 0xc76c51a3, 0xd192e819, 0xd6990624, 0xf40e3585, 0x106aa070,
    0x19a4c116, 0x1e376c08, 0x2748774c, 0x34b0bcb5, 0x391c0cb3, 0x4ed8aa4a, 0x5b9cca4f, 0x682e6ff3,
    0x748f82ee, 0x78a5636f, 0x84c87814, 0x8cc70208, 0x90befffa, 0xa4506ceb, 0xbef9a3f7, 0xc67178f2};

int g_force_portable = 0;

inline uint32_t rotr(uint32_t x, int n) { return (x >> n) | (x << (32 - n)); }

// The compression function written out from the standard: message schedule, then 64 rounds.
void blocks_portable(uint32_t h[8], const uint8_t* p, size_t nblk)
{
    for (; nblk; --nblk, p += 64) {
        uint32_t w[64];
        for (int t = 0; t < 16; ++t)
            w[t] = (uint32_t)p[4 * t] << 24 | (uint32_t)p[4 * t + 1] << 16 | (uint32_t)p[4 * t + 2] << 8 | p[4 * t + 3];
        for (int t = 16; t < 64; ++t) {
            const uint32_t s0 = rotr(w[t - 15], 7) ^ rotr(w[t - 15], 18) ^ (w[t - 15] >> 3);
            const uint32_t s1 = rotr(w[t - 2], 17) ^ rotr(w[t - 2], 19) ^ (w[t - 2] >> 10);
            w[t] = w[t - 16] + s0 + w[t - 7] + s1;
        }
        uint32_t a = h[0], b = h[1], c = h[2], d = h[3], e = h[4], f = h[5], g = h[6], k = h[7];
        for (int t = 0; t < 64; ++t) {
            const uint32_t S1 = rotr(e, 6) ^ rotr(e, 11) ^ rotr(e, 25);
            const uint32_t ch = (e & f) ^ (~e & g);
            const uint32_t t1 = k + S1 + ch + kK[t] + w[t];
            const uint32_t S0 = rotr(a, 2) ^ rotr(a, 13) ^ rotr(a, 22);
            const uint32_t mj = (a & b) ^ (a & c) ^ (b & c);
            const uint32_t t2 = S0 + mj;
            k = g; g = f; f = e; e = d + t1; d = c; c = b; b = a; a = t1 + t2;
        }
        h[0] += a; h[1] += b; h[2] += c; h[3] += d; h[4] += e; h[5] += f; h[6] += g; h[7] += k;
    }
}

// The same function on the x86 SHA extensions: the state lives in two registers as (A,B,E,F) and
// (C,D,G,H); a group of four rounds takes one four-word slice W_g of the schedule, and for g >= 4
// W_g = msg2( msg1(W_{g-4}, W_{g-3}) + (W_{g-2}, W_{g-1} shifted by one word), W_{g-1} ).
__attribute__((target("sha,sse4.1,ssse3"))) void blocks_shaext(uint32_t h[8], const uint8_t* p, size_t nblk)
{
    const __m128i bswap = _mm_set_epi64x(0x0c0d0e0f08090a0bLL, 0x0405060700010203LL);
    __m128i t = _mm_loadu_si128(reinterpret_cast<const __m128i*>(h));       // D C B A (high .. low)
    __m128i s1 = _mm_loadu_si128(reinterpret_cast<const __m128i*>(h + 4));  // H G F E
    t = _mm_shuffle_epi32(t, 0xB1);                                         // C D A B
    s1 = _mm_shuffle_epi32(s1, 0x1B);                                       // E F G H
    __m128i s0 = _mm_alignr_epi8(t, s1, 8);                                 // A B E F
    s1 = _mm_blend_epi16(s1, t, 0xF0);                                      // C D G H
    for (; nblk; --nblk, p += 64) {
        const __m128i save0 = s0, save1 = s1;
        __m128i w[4];
        for (int g = 0; g < 16; ++g) {
            __m128i wg;
            if (g < 4) {
                wg = _mm_shuffle_epi8(_mm_loadu_si128(reinterpret_cast<const __m128i*>(p + 16 * g)), bswap);
            } else {
                __m128i x = _mm_sha256msg1_epu32(w[g & 3], w[(g + 1) & 3]);
                x = _mm_add_epi32(x, _mm_alignr_epi8(w[(g + 3) & 3], w[(g + 2) & 3], 4));
                wg = _mm_sha256msg2_epu32(x, w[(g + 3) & 3]);
            }
            w[g & 3] = wg;
            __m128i m = _mm_add_epi32(wg, _mm_loadu_si128(reinterpret_cast<const __m128i*>(kK + 4 * g)));
            s1 = _mm_sha256rnds2_epu32(s1, s0, m);
            m = _mm_shuffle_epi32(m, 0x0E);
            s0 = _mm_sha256rnds2_epu32(s0, s1, m);
        }
        s0 = _mm_add_epi32(s0, save0);
        s1 = _mm_add_epi32(s1, save1);
    }
    t = _mm_shuffle_epi32(s0, 0x1B);     // F E B A
    s1 = _mm_shuffle_epi32(s1, 0xB1);    // D C H G
    s0 = _mm_blend_epi16(t, s1, 0xF0);   // D C B A
    s1 = _mm_alignr_epi8(s1, t, 8);      // H G F E
    _mm_storeu_si128(reinterpret_cast<__m128i*>(h), s0);
    _mm_storeu_si128(reinterpret_cast<__m128i*>(h + 4), s1);
}

void blocks(uint32_t h[8], const uint8_t* p, size_t nblk)
{
    static const int have_sha = __builtin_cpu_supports("sha") && __builtin_cpu_supports("sse4.1");
    if (have_sha && !g_force_portable)
        blocks_shaext(h, p, nblk);
    else
        blocks_portable(h, p, nblk);
}

}  // namespace

extern "C" int det_sha256_init(det_sha256_ctx* c)
{
    if (!c) return DET_EINVAL;
    static const uint32_t iv[8] = {0x6a09e667, 0xbb67ae85, 0x3c6ef372, 0xa54ff53a,
                                   0x510e527f, 0x9b05688c, 0x1f83d9ab, 0x5be0cd19};
    memcpy(c->h, iv, sizeof(iv));
    c->nbytes = 0;
    c->fill = 0;
    return DET_OK;
}

extern "C" int det_sha256_update(det_sha256_ctx* c, const void* data, size_t bytes)
{
    if (!c || (!data && bytes) || c->fill >= 64) return DET_EINVAL;
    const uint8_t* p = static_cast<const uint8_t*>(data);
    c->nbytes += bytes;
    if (c->fill) {
        const size_t take = bytes < 64 - c->fill ? bytes : 64 - c->fill;
        memcpy(c->buf + c->fill, p, take);
        c->fill += (uint32_t)take;
        p += take;
        bytes -= take;
        if (c->fill < 64) return DET_OK;
        blocks(c->h, c->buf, 1);
        c->fill = 0;
    }
    blocks(c->h, p, bytes / 64);
    p += bytes & ~(size_t)63;
    bytes &= 63;
    memcpy(c->buf, p, bytes);
    c->fill = (uint32_t)bytes;
    return DET_OK;
}

extern "C" int det_sha256_final(det_sha256_ctx* c, uint8_t digest[32])
{
    if (!c || !digest || c->fill >= 64) return DET_EINVAL;
    const uint64_t bits = c->nbytes * 8;
    uint8_t pad[128];
    memset(pad, 0, sizeof(pad));
    memcpy(pad, c->buf, c->fill);
    pad[c->fill] = 0x80;
    const size_t total = c->fill < 56 ? 64 : 128;
    for (int i = 0; i < 8; ++i) pad[total - 1 - i] = (uint8_t)(bits >> (8 * i));
    blocks(c->h, pad, total / 64);
    for (int i = 0; i < 8; ++i) {
        digest[4 * i] = (uint8_t)(c->h[i] >> 24);
        digest[4 * i + 1] = (uint8_t)(c->h[i] >> 16);
        digest[4 * i + 2] = (uint8_t)(c->h[i] >> 8);
        digest[4 * i + 3] = (uint8_t)c->h[i];
    }
    c->fill = 64;  // spent: a further update or final is an error
    return DET_OK;
}

extern "C" int det_commit_sha256(const void* prompt, size_t prompt_bytes, const void* logits, size_t logits_bytes,
                                 const void* tokens, size_t tokens_bytes, uint8_t digest[32])
{
    det_sha256_ctx c;
    int rc = det_sha256_init(&c);
    if (rc == DET_OK) rc = det_sha256_update(&c, prompt, prompt_bytes);
    if (rc == DET_OK) rc = det_sha256_update(&c, logits, logits_bytes);
    if (rc == DET_OK) rc = det_sha256_update(&c, tokens, tokens_bytes);
    if (rc == DET_OK) rc = det_sha256_final(&c, digest);
    return rc;
}

extern "C" int det_sha256_force_portable(int on)
{
    g_force_portable = on != 0;
    return DET_OK;
}
