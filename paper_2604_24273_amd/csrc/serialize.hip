// State-to-token front end, serialize(s_t) of the paper's Sec. 3.1, Eq. 3: host code only (the paper
// spends 1.2 ms of a 24.8 ms step here, Sec. 5.2; nothing in it is worth a kernel).
//
// A state vector becomes the text "state:" + " v" per dimension, v the value clamped to [-9.9, 9.9]
// with one decimal (correctly rounded from the exact fp32 value, exact ties to the even digit, zero
// without a sign, NaN as zero), and the text becomes token ids of a stand-in vocabulary of 457
// entries: 0 begin-of-state, 1 "state:", 2 .. 200 the number strings " -9.9" .. " 9.9", 201 .. 456 the
// single bytes.  A state of n dimensions is n + 2 tokens (the paper reports 15 - 40 tokens for 17 - 27
// dimensions).  The backbone's own tokenizer is not part of this library; a caller that has it feeds
// its ids to encoder_forward_packed directly.
#include <cstring>

#include "common.hpp"

namespace brl {
namespace {

constexpr int SER_BOS = 0, SER_STATE = 1, SER_NUM0 = 2 + 99 /* id of " 0.0" */, SER_BYTE0 = 201;
const char SER_PREFIX[] = "state:";
constexpr int SER_PREFIX_LEN = 6;

// tenths of the clamped value, from the bits of the float: |x| = M * 2^E exactly, so 10 |x| = (10 M) >> -E
// with a remainder that decides the rounding - no floating-point operation, no locale
int tenths_of(float x) {
    uint32_t u;
    memcpy(&u, &x, 4);
    const bool neg = (u >> 31) != 0;
    const uint32_t ex = (u >> 23) & 0xffu, man = u & 0x7fffffu;
    if (ex == 0xffu) return man ? 0 : (neg ? -99 : 99);            // NaN -> 0, infinities clamp
    const float ax = neg ? -x : x;
    if (ax >= 9.9f) return neg ? -99 : 99;                          // fp32(9.9) and above render as 9.9
    const uint64_t M = ex ? (uint64_t)(man | 0x800000u) : (uint64_t)man;
    const int E = (ex ? (int)ex : 1) - 150;                        // |x| = M * 2^E, here E <= -20
    const uint64_t t = M * 10u;                                     // < 2^28
    const int sh = -E;
    uint64_t q = 0;
    if (sh < 63) {
        q = t >> sh;
        const uint64_t rem = t & (((uint64_t)1 << sh) - 1), half = (uint64_t)1 << (sh - 1);
        if (rem > half || (rem == half && (q & 1u))) ++q;
    }
    const int m = (int)q;
    return neg ? -m : m;
}

// " d.d" or " -d.d" (zero unsigned); returns the number of bytes written
int put_number(int m, char* out) {
    int n = 0;
    out[n++] = ' ';
    if (m < 0) { out[n++] = '-'; m = -m; }
    out[n++] = (char)('0' + m / 10);
    out[n++] = '.';
    out[n++] = (char)('0' + m % 10);
    return n;
}

inline bool is_digit(unsigned char c) { return c >= '0' && c <= '9'; }

}  // namespace
}  // namespace brl

using namespace brl;

extern "C" {

size_t brl_serialize_text(const float* state, int n_dims, char* text_out, size_t cap) {
    if (!state || n_dims < 0) return 0;
    size_t need = SER_PREFIX_LEN;
    for (int i = 0; i < n_dims; ++i) need += tenths_of(state[i]) < 0 ? 5 : 4;
    if (!text_out || cap < need + 1) return need;                  // the caller asks again with need + 1 bytes
    memcpy(text_out, SER_PREFIX, SER_PREFIX_LEN);
    size_t p = SER_PREFIX_LEN;
    for (int i = 0; i < n_dims; ++i) p += (size_t)put_number(tenths_of(state[i]), text_out + p);
    text_out[p] = '\0';
    return need;
}

int brl_tokenize(const char* text, size_t n_bytes, int32_t* ids_out, int max_ids, int* n_ids) {
    BRL_REQUIRE((text || n_bytes == 0) && n_ids && (ids_out || max_ids == 0) && max_ids >= 0, "tokenize: null pointer");
    const unsigned char* s = reinterpret_cast<const unsigned char*>(text);
    int n = 0;
    auto emit = [&](int id) {
        if (n < max_ids) ids_out[n] = id;
        ++n;
    };
    emit(SER_BOS);
    size_t p = 0;
    while (p < n_bytes) {
        const size_t left = n_bytes - p;
        if (left >= (size_t)SER_PREFIX_LEN && memcmp(s + p, SER_PREFIX, SER_PREFIX_LEN) == 0) {
            emit(SER_STATE);
            p += SER_PREFIX_LEN;
        } else if (left >= 5 && s[p] == ' ' && s[p + 1] == '-' && is_digit(s[p + 2]) && s[p + 3] == '.' && is_digit(s[p + 4]) &&
                   (s[p + 2] != '0' || s[p + 4] != '0')) {
            emit(SER_NUM0 - (10 * (s[p + 2] - '0') + (s[p + 4] - '0')));
            p += 5;
        } else if (left >= 4 && s[p] == ' ' && is_digit(s[p + 1]) && s[p + 2] == '.' && is_digit(s[p + 3])) {
            emit(SER_NUM0 + 10 * (s[p + 1] - '0') + (s[p + 3] - '0'));
            p += 4;
        } else {
            emit(SER_BYTE0 + s[p]);
            p += 1;
        }
    }
    *n_ids = n;
    if (n > max_ids) {
        set_error("tokenize: %d tokens, room for %d", n, max_ids);
        return BRL_ENOSPC;
    }
    return BRL_OK;
}

int serialize_states(const float* states, int B, int n_dims, int vocab, int32_t* ids_out, int32_t* cu_seqlens_out) {
    BRL_REQUIRE(states && ids_out && cu_seqlens_out, "serialize_states: null pointer");
    BRL_REQUIRE(B >= 1 && n_dims >= 1, "serialize_states: B = %d, n_dims = %d", B, n_dims);
    BRL_REQUIRE(vocab >= BRL_SERIALIZE_VOCAB, "serialize_states: the encoder's vocabulary (%d) is smaller than the %d ids used",
                vocab, BRL_SERIALIZE_VOCAB);
    BRL_REQUIRE((long long)B * (n_dims + 2) < (1ll << 31), "serialize_states: too many tokens");
    int32_t* out = ids_out;
    cu_seqlens_out[0] = 0;
    for (int b = 0; b < B; ++b) {
        const float* s = states + (size_t)b * n_dims;
        *out++ = SER_BOS;
        *out++ = SER_STATE;
        for (int i = 0; i < n_dims; ++i) *out++ = SER_NUM0 + tenths_of(s[i]);
        cu_seqlens_out[b + 1] = (int32_t)(out - ids_out);
    }
    return BRL_OK;
}

}  // extern "C"
